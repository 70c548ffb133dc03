"""GPU parity, part 2: the matmul through the C ABI against the oracle, within
|C_gpu - C_ref| <= 1e-2 + 5e-3 |C_ref| elementwise; exact where the arithmetic
admits one answer (one-hot rows, small integers)."""
import numpy as np
import pytest
import torch

from oracle import qgemm_oracle as O
from paper_2504_12984_amd import workloads as WL
from gpu_util import Prepared, assert_c_close, bits_of, to_f64

pytestmark = pytest.mark.gpu

U, I, F = WL.KIND_UINT, WL.KIND_INT, WL.KIND_FLOAT
FLOATS = [(3, 1, 1), (4, 2, 1), (5, 2, 2), (6, 3, 2), (7, 3, 3), (8, 4, 3)]


@pytest.fixture(autouse=True)
def _reset_knobs():
    from paper_2504_12984_amd import binding as B
    yield
    for k in range(4):
        B.qg_set_knob(k, 0)


def test_config1_tiny_gemv_full():
    P = Prepared(WL.cfg1())
    assert_c_close(P.gpu_c(), P.oracle_c(), "cfg1")


@pytest.mark.parametrize("M", [1, 2, 3, 4, 15, 16, 17, 31, 32, 33, 48, 64])
def test_small_m_every_row_count(M):
    # several tiles in N (3 strips), several chunks per wavefront and a ragged
    # split of K across the 8 wavefronts (K/128 = 11)
    case = WL.Case(f"small_M{M}", M, 1408, 192, U, 4, group=128, zero=8, seed=8000 + M)
    P = Prepared(case)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("bits", range(1, 9))
@pytest.mark.parametrize("kind", [U, I])
def test_small_m_integer_types(kind, bits, act):
    sdt = "f16" if act == "f16" else "bf16"
    case = WL.Case(f"small_{kind}_{bits}_{act}", 16, 2048, 256, kind, bits, group=64 if bits % 2 else 128,
                   act=act, scale_dtype=sdt, zero=(1 << (bits - 1)) if kind == U else None, seed=8100 + bits)
    P = Prepared(case)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("bits,e,m", FLOATS)
def test_small_m_float_types(bits, e, m, act):
    case = WL.Case(f"small_f{bits}_{act}", 5, 1024, 128, F, bits, e, m, group=1024, act=act, scale_dtype="f16",
                   zero=None, scale_lo=0.01, scale_hi=0.1, seed=8200 + bits)
    P = Prepared(case)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("splitk", [1, 2, 3, 8, 11])
def test_split_k_factors_agree_with_oracle_and_leave_counters_clean(splitk):
    from paper_2504_12984_amd import binding as B
    case = WL.Case(f"splitk_{splitk}", 7, 1408, 320, U, 3, group=128, zero=4, seed=8300)
    P = Prepared(case)
    ref = P.oracle_c()
    B.qg_set_knob(1, splitk)
    first = P.gpu_c()
    assert_c_close(first, ref, case.name)
    # a second call must see zeroed arrival counters and give identical bits
    second = P.gpu_c()
    assert np.array_equal(bits_of(first), bits_of(second))


@pytest.mark.parametrize("splitk", [1, 3])
@pytest.mark.parametrize("variant", [10, 11, 12, 14, 15, 16])
@pytest.mark.parametrize("M", [1, 16])
def test_every_wavefront_arrangement_of_the_streaming_kernel(M, variant, splitk):
    # 8, 4 or 16 wavefronts on one strip, or 8 / 16 on two strips
    from paper_2504_12984_amd import binding as B
    case = WL.Case(f"arr_{M}_{variant}_{splitk}", M, 1408, 512, I, 3, group=128, zero=None, seed=8350 + M)
    P = Prepared(case)
    B.qg_set_knob(3, variant)
    B.qg_set_knob(1, splitk)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("M,variant", [(17, 21), (32, 26), (30, 26), (33, 41), (64, 46), (50, 46)])
def test_two_strip_arrangements_with_several_row_tiles(M, variant):
    from paper_2504_12984_amd import binding as B
    case = WL.Case(f"arr2_{M}_{variant}", M, 1152, 256, U, 6, group=128, act="bf16", scale_dtype="bf16",
                   zero=31, seed=8360 + M)
    P = Prepared(case)
    B.qg_set_knob(3, variant)
    for splitk in (1, 2):
        B.qg_set_knob(1, splitk)
        assert_c_close(P.gpu_c(), P.oracle_c(), f"{case.name} splitk={splitk}")


def test_one_hot_rows_return_weight_rows_bit_exactly():
    # ties the matmul to the bit-exact de-quantisation: fp32 accumulation of a
    # single non-zero product and one rounding reproduce the weight itself
    for act in ("f16", "bf16"):
        case = WL.Case(f"onehot_{act}", 16, 512, 128, U, 5, group=128, act=act,
                       scale_dtype="f16", zero=16, seed=8400)
        inp = WL.make_inputs(case)
        rows = np.array([0, 1, 7, 8, 31, 32, 127, 128, 129, 255, 256, 300, 383, 384, 510, 511])
        A = torch.zeros((16, 512), dtype=inp["A"].dtype)
        A[torch.arange(16), torch.from_numpy(rows)] = 1.0
        inp["A"] = A
        P = Prepared(case, inp)
        _, wbits = P.oracle_w()
        assert np.array_equal(bits_of(P.gpu_c()), wbits[rows]), act


def test_uint8_unit_scale_small_integers_is_exact():
    case = WL.Case("int_exact", 16, 256, 128, U, 8, group=256, zero=None, seed=8500)
    inp = WL.make_inputs(case)
    rng = np.random.default_rng(1)
    inp["A"] = torch.from_numpy(rng.integers(-1, 2, size=(16, 256)).astype(np.float32)).to(torch.float16)
    inp["codes"] = rng.integers(0, 8, size=(256, 128), dtype=np.uint8)
    inp["scales"] = torch.ones((1, 128), dtype=torch.float16)
    P = Prepared(case, inp)
    want = to_f64(inp["A"]).astype(np.int64) @ inp["codes"].astype(np.int64)
    assert np.abs(want).max() < 2048
    assert np.array_equal(to_f64(P.gpu_c()), want.astype(np.float64))


def test_empty_m_and_bad_arguments():
    from paper_2504_12984_amd import binding as B
    case = WL.Case("edge", 1, 128, 64, U, 4, group=128, zero=8, seed=8600)
    P = Prepared(case)
    A0 = torch.empty((0, 128), dtype=torch.float16, device="cuda")
    assert P.gpu_c(A0).shape == (0, 64)
    with pytest.raises(B.QgError):      # group 16 is no group size of this library
        s = torch.ones((8, 64), dtype=torch.float16, device="cuda")
        B.qgemm(P.d_A, P.d_packed, s, None, P.wtype, 16, 64)


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("M", [1, 16, 20, 40, 64, 65, 150])
def test_group_size_32(M, act):
    # four groups per 128-row chunk: streaming kernel up to 64 rows, tiled kernel beyond (and
    # forced, at every tile height); the second layout's kernel has no such variant and says so
    from paper_2504_12984_amd import binding as B
    kind, bits = (U, 4) if M % 2 == 0 else (I, 3)
    sdt = "f16" if act == "f16" else "bf16"
    case = WL.Case(f"g32_{M}_{act}", M, 640, 192, kind, bits, group=32, act=act, scale_dtype=sdt,
                   zero=8 if kind == U else None, seed=8610 + M)
    P = Prepared(case)
    ref = P.oracle_c()
    assert_c_close(P.gpu_c(), ref, case.name)
    plan = B.qg_plan(P.wtype, 32, M, case.N, case.K, act=B.QG_F16 if act == "f16" else B.QG_BF16)
    assert plan["path"] == (1 if M <= 64 else 2)
    B.qg_set_knob(0, 2)
    for bm in (64, 128, 256):
        B.qg_set_knob(2, bm)
        assert_c_close(P.gpu_c(), ref, f"{case.name} tiled {bm}")
    B.qg_set_knob(0, 3)
    assert_c_close(P.gpu_c(), ref, f"{case.name} row blocks")
    B.qg_set_knob(0, 0); B.qg_set_knob(2, 0)
    with pytest.raises(B.QgError):
        P.gpu_c(layout=1)


@pytest.mark.parametrize("bits", [1, 3, 5, 8])
def test_group_size_32_tiled_path_types_and_odd_chunk_counts(bits):
    from paper_2504_12984_amd import binding as B
    # 7 chunks (odd: the padding chunk), several row tiles, idle wavefronts (N = 192), split-K
    case = WL.Case(f"g32_tiled_{bits}", 300, 896, 192, U, bits, group=32, act="f16" if bits % 2 else "bf16",
                   scale_dtype="f16", zero=(1 << bits) // 2, seed=8640 + bits)
    P = Prepared(case)
    ref = P.oracle_c()
    assert_c_close(P.gpu_c(), ref, case.name)
    B.qg_set_knob(0, 2); B.qg_set_knob(2, 64); B.qg_set_knob(1, 2)
    assert_c_close(P.gpu_c(), ref, case.name + " split")


def test_group_size_32_split_k_and_float_weights():
    from paper_2504_12984_amd import binding as B
    case = WL.Case("g32_f6", 7, 1408, 320, F, 6, 3, 2, group=32, act="bf16", scale_dtype="f16", zero=None,
                   scale_lo=0.01, scale_hi=0.1, seed=8630)
    P = Prepared(case)
    ref = P.oracle_c()
    for splitk in (0, 3):
        B.qg_set_knob(1, splitk)
        assert_c_close(P.gpu_c(), ref, f"{case.name} splitk {splitk}")


# ------------------------------------------------------------------ tiled path
@pytest.mark.parametrize("bm", [64, 128, 256])
@pytest.mark.parametrize("M,K,N", [(200, 512, 256), (257, 384, 320), (65, 128, 64), (512, 1024, 512)])
def test_tiled_path_ragged_shapes(M, K, N, bm):
    from paper_2504_12984_amd import binding as B
    case = WL.Case(f"tiled_{M}_{K}_{N}_{bm}", M, K, N, U, 5, group=64, act="bf16", scale_dtype="bf16",
                   zero=16, seed=8700 + M)
    P = Prepared(case)
    B.qg_set_knob(0, 2)                 # the tiled kernel, whatever the automatic choice would be
    B.qg_set_knob(2, bm)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("act", ["f16", "bf16"])
@pytest.mark.parametrize("kind,bits,e,m", [(U, 1, 0, 0), (I, 2, 0, 0), (U, 3, 0, 0), (I, 4, 0, 0), (U, 6, 0, 0),
                                           (I, 7, 0, 0), (U, 8, 0, 0), (F, 4, 2, 1), (F, 6, 3, 2), (F, 8, 4, 3)])
def test_tiled_path_weight_types(kind, bits, e, m, act):
    from paper_2504_12984_amd import binding as B
    case = WL.Case(f"tiled_t{kind}_{bits}_{act}", 130, 640, 192, kind, bits, e, m, group=128, act=act,
                   scale_dtype="f16", zero=(1 << (bits - 1)) if kind == U else None, seed=8800 + bits)
    P = Prepared(case)
    B.qg_set_knob(0, 2)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("bm", [64, 128])
@pytest.mark.parametrize("splitk", [2, 3, 4, 11])
@pytest.mark.parametrize("M,K,N,group", [(40, 1408, 320, 128), (64, 1024, 256, 64), (150, 896, 192, 128)])
def test_tiled_path_split_k(M, K, N, group, splitk, bm):
    # slabs of an even number of chunks with a shorter (odd: 11 chunks in slabs of 4, 7 in
    # slabs of 4) last slab, idle wavefronts (N not a multiple of 256), rows past M, more
    # slabs asked for than there are chunk pairs; the second call must find the arrival
    # counters at zero and give identical bits
    from paper_2504_12984_amd import binding as B
    case = WL.Case(f"tiled_splitk_{M}_{K}_{N}_{splitk}_{bm}", M, K, N, U, 4, group=group, act="bf16",
                   scale_dtype="bf16", zero=8, seed=8870 + M + splitk)
    P = Prepared(case)
    ref = P.oracle_c()
    B.qg_set_knob(0, 2)
    B.qg_set_knob(1, splitk)
    B.qg_set_knob(2, bm)
    first = P.gpu_c()
    assert_c_close(first, ref, case.name)
    second = P.gpu_c()
    assert np.array_equal(bits_of(first), bits_of(second))


@pytest.mark.parametrize("bm", [64, 128, 256])
@pytest.mark.parametrize("bits", [1, 3, 4, 7, 8])
def test_tiled_path_fp16_two_groups_per_chunk(bits, bm):
    # group 64 puts two sets of scales / zero-points in every 128-row chunk
    from paper_2504_12984_amd import binding as B
    case = WL.Case(f"tiled_g64_{bits}_{bm}", 130, 640, 192, U, bits, group=64, act="f16", scale_dtype="f16",
                   zero=1 << (bits - 1), seed=8850 + bits)
    P = Prepared(case)
    B.qg_set_knob(0, 2)
    B.qg_set_knob(2, bm)
    assert_c_close(P.gpu_c(), P.oracle_c(), case.name)


@pytest.mark.parametrize("M", [65, 100, 128, 129, 192])
def test_moderate_m_on_few_tiles_automatic_row_blocks_and_tiled(M):
    # the automatic choice, the streaming kernel over blocks of 64 rows (ragged last block) and the tiled kernel
    from paper_2504_12984_amd import binding as B
    case = WL.Case(f"blocks_{M}", M, 1152, 320, I, 5, group=128, act="bf16", scale_dtype="f16", zero=None,
                   seed=8870 + M)
    P = Prepared(case)
    ref = P.oracle_c()
    assert_c_close(P.gpu_c(), ref, case.name + " auto")
    B.qg_set_knob(0, 3)
    assert_c_close(P.gpu_c(), ref, case.name + " forced")
    B.qg_set_knob(0, 2)
    assert_c_close(P.gpu_c(), ref, case.name + " tiled")


def test_both_paths_agree_with_the_oracle_on_the_same_small_problem():
    from paper_2504_12984_amd import binding as B
    case = WL.Case("both_paths", 48, 768, 256, U, 6, group=128, act="bf16", scale_dtype="bf16", zero=32, seed=8900)
    P = Prepared(case)
    ref = P.oracle_c()
    for path in (1, 2):
        B.qg_set_knob(0, path)
        assert_c_close(P.gpu_c(), ref, f"path {path}")


def test_tiled_path_one_hot_rows_bit_exact():
    from paper_2504_12984_amd import binding as B
    case = WL.Case("tiled_onehot", 256, 256, 128, I, 6, group=128, act="bf16", scale_dtype="f16", zero=None, seed=8950)
    inp = WL.make_inputs(case)
    A = torch.zeros((256, 256), dtype=torch.bfloat16)
    A[torch.arange(256), torch.arange(256)] = 1.0
    inp["A"] = A
    P = Prepared(case, inp)
    _, wbits = P.oracle_w()
    B.qg_set_knob(0, 2)
    assert np.array_equal(bits_of(P.gpu_c()), wbits)


@pytest.mark.parametrize("layout", [0, 1])
def test_tiled_path_split_into_whole_rounds_plus_remainder(layout):
    # 2 x 140 tiles of 256 rows: one whole round of 256 workgroups (128 column tiles) and a
    # second launch for the last 12 column tiles; columns from both parts are checked
    case = WL.Case(f"rounds_{layout}", 512, 256, 35840, U, 4, group=128, act="bf16", scale_dtype="bf16",
                   zero=8, seed=9050)
    P = Prepared(case)
    cols = np.concatenate([np.arange(0, 64), np.arange(32704, 32832), np.arange(35776, 35840),
                           np.random.default_rng(5).integers(0, 35840, size=64)])
    got = P.gpu_c(layout=layout)
    assert_c_close(got[:, torch.from_numpy(cols).cuda()], P.oracle_c(cols=cols), case.name)


@pytest.mark.parametrize("kernel", ["streaming", "tiled64", "tiled128"])
def test_split_k_workspace_reused_by_different_inputs_back_to_back(kernel):
    # Calls with DIFFERENT inputs go through the same workspace slots and arrival counters
    # one after the other on one stream with nothing in between (X, Y, Z, X, Y; X and Y have
    # the same shape, Z another one whose tiles overlap theirs): the last arriver of a call
    # must sum this call's partial tiles, never what an earlier call left in the workspace
    # or in a cache.  Every result is compared with the oracle.
    from paper_2504_12984_amd import binding as B
    if kernel == "streaming":
        mk = lambda tag, K, N, seed: WL.Case(f"xyx_s_{tag}", 16, K, N, U, 4, group=128, zero="random", seed=seed)
        B.qg_set_knob(0, 1); B.qg_set_knob(1, 4)
    else:
        mk = lambda tag, K, N, seed: WL.Case(f"xyx_t_{tag}", 100, K, N, U, 4, group=128, act="bf16",
                                             scale_dtype="bf16", zero="random", seed=seed)
        B.qg_set_knob(0, 2); B.qg_set_knob(1, 4); B.qg_set_knob(2, 64 if kernel == "tiled64" else 128)
    X, Y, Z = Prepared(mk("X", 2048, 512, 9200)), Prepared(mk("Y", 2048, 512, 9201)), Prepared(mk("Z", 1536, 320, 9202))
    refs = {id(P): P.oracle_c() for P in (X, Y, Z)}
    assert not np.allclose(refs[id(X)], refs[id(Y)])
    order = [X, Y, Z, X, Y]
    torch.cuda.synchronize()
    outs = [P.gpu_c() for P in order]                # enqueued back to back, no synchronisation
    torch.cuda.synchronize()
    for i, (P, C) in enumerate(zip(order, outs)):
        assert_c_close(C, refs[id(P)], f"{P.case.name} call {i}")
    assert np.array_equal(bits_of(outs[0]), bits_of(outs[3])) and np.array_equal(bits_of(outs[1]), bits_of(outs[4]))


# ------------------------------------------------------------------ binding extras
def test_split_k_calls_on_two_streams_keep_separate_workspaces():
    # a streaming split-K matmul and a tiled split-K matmul enqueued alternately on two
    # streams (free to overlap) must give the bits they give alone on the default stream
    from paper_2504_12984_amd import binding as B
    small = WL.Case("streams_small", 16, 8192, 2048, U, 4, group=128, zero=8, seed=8950)
    mid = WL.Case("streams_mid", 128, 8192, 2048, U, 4, group=128, act="bf16", scale_dtype="bf16", zero=8, seed=8951)
    P1, P2 = Prepared(small), Prepared(mid)
    assert B.qg_plan(P1.wtype, 128, 16, 2048, 8192)["splitk"] > 1
    assert B.qg_plan(P2.wtype, 128, 128, 2048, 8192, act=B.QG_BF16)["splitk"] > 1
    alone1, alone2 = P1.gpu_c(), P2.gpu_c()
    assert_c_close(alone1, P1.oracle_c(), small.name)
    assert_c_close(alone2, P2.oracle_c(), mid.name)
    torch.cuda.synchronize()
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    outs = []
    for _ in range(10):
        with torch.cuda.stream(s1):
            outs.append((P1.gpu_c(), alone1))
        with torch.cuda.stream(s2):
            outs.append((P2.gpu_c(), alone2))
    torch.cuda.synchronize()
    for got, want in outs:
        assert np.array_equal(bits_of(got), bits_of(want))


def test_group_zero_means_one_scale_per_output_column():
    from paper_2504_12984_amd import binding as B
    from gpu_util import ACT
    case = WL.Case("group0", 20, 512, 128, U, 4, group=512, act="bf16", scale_dtype="bf16", zero=8, seed=8960)
    P = Prepared(case)
    ref = P.oracle_c()
    C0 = B.qgemm(P.d_A, P.packed(0), P.d_scales, P.d_zeros, P.wtype, 0, case.N)
    assert_c_close(C0, ref, case.name)
    assert np.array_equal(bits_of(C0), bits_of(P.gpu_c()))
    W0 = B.qdequant(P.packed(0), P.d_scales, P.d_zeros, P.wtype, ACT[case.act], 0, case.K, case.N)
    assert np.array_equal(bits_of(W0), bits_of(P.gpu_w(0)))


def test_graph_capture_of_qgemm_calls_replays_to_the_eager_bits():
    # a streaming split-K call, a tiled split-K call and a plain tiled call captured in one HIP
    # graph; every replay (with eager work and synchronisations in between) must reproduce the
    # eager results bit for bit -- arrival counters and workspaces are left ready by each launch.
    # The first call on a stream allocates its workspace, so the calls run once eagerly on the
    # capture stream before the capture.
    from paper_2504_12984_amd import binding as B
    cases = [WL.Case("graph_small", 16, 8192, 2048, U, 4, group=128, zero=8, seed=8970),
             WL.Case("graph_mid", 128, 8192, 2048, U, 4, group=128, act="bf16", scale_dtype="bf16", zero=8, seed=8971),
             WL.Case("graph_big", 300, 512, 1024, I, 5, group=64, act="bf16", scale_dtype="f16", zero=None, seed=8972)]
    Ps = [Prepared(c) for c in cases]
    eager = [P.gpu_c() for P in Ps]
    for P, C in zip(Ps, eager):
        assert_c_close(C, P.oracle_c(), P.case.name)
    outs = [torch.empty_like(C) for C in eager]
    torch.cuda.synchronize()
    side = torch.cuda.Stream()

    def enqueue():
        for P, out in zip(Ps, outs):
            B.qgemm(P.d_A, P.packed(0), P.d_scales, P.d_zeros, P.wtype, P.case.group, P.case.N, out=out)

    with torch.cuda.stream(side):
        enqueue()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        enqueue()
    for rep in range(3):
        for out in outs:
            out.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for out, C, P in zip(outs, eager, Ps):
            assert np.array_equal(bits_of(out), bits_of(C)), f"{P.case.name} replay {rep}"


def test_bound_call_gives_the_same_bits_as_the_plain_call_and_checks_its_arguments():
    from paper_2504_12984_amd import binding as B
    case = WL.Case("bound", 7, 640, 192, U, 4, group=128, zero=8, seed=9100)
    P = Prepared(case)
    want = P.gpu_c()
    out = torch.empty_like(want)
    call = B.BoundQgemm(P.d_A, P.d_packed, P.d_scales, P.d_zeros, P.wtype, case.group, case.N, out)
    for _ in range(3):                               # repeated calls reuse the marshalled arguments
        got = call()
        assert got is out
        assert np.array_equal(bits_of(got), bits_of(want))
    with pytest.raises(ValueError):                  # output of the wrong shape
        B.BoundQgemm(P.d_A, P.d_packed, P.d_scales, P.d_zeros, P.wtype, case.group, case.N, out[:, :64])
    with pytest.raises(ValueError):                  # scales of the wrong shape
        B.BoundQgemm(P.d_A, P.d_packed, P.d_scales[:2], P.d_zeros, P.wtype, case.group, case.N, out)


def test_measurement_probes_run_and_report_their_flops():
    from paper_2504_12984_amd import binding as B
    sink = torch.zeros(1024, dtype=torch.float32, device="cuda")
    buf = torch.ones(1 << 22, dtype=torch.uint8, device="cuda")
    probe = B.qg_probe_stream_read(buf, sink)
    probe()
    flops = B.qg_probe_mfma(True, True, 10, 1, sink)
    assert flops == 8.0 * 32768.0 * 10 * 4.0 * 256.0
    flops2 = B.qg_probe_mfma(False, False, 5, 2, sink)
    assert flops2 == 8.0 * 32768.0 * 5 * 4.0 * 512.0
    torch.cuda.synchronize()
    assert float(sink.abs().sum()) == 0.0            # the probes never write their sink
    with pytest.raises(B.QgError):
        B.qg_probe_mfma(True, True, 0, 1, sink)

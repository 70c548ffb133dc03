"""GPU test of qgemm_noalloc, the entry point that allocates nothing: its split-K scratch
is one fixed array in device memory that belongs to the loaded library.

Through the C ABI, calls in a row on one stream -- the later ones smaller, so that they
find the earlier ones' partial sums and (zeroed) counters in the shared array -- must give
the bits qgemm gives for the same arguments (same kernels, same plan) and agree with the
oracle within |C_gpu - C_ref| <= 1e-2 + 5e-3 |C_ref|.  Device memory in use must not grow
across the calls, and a request beyond the array must be refused with a clear message.
"""
import numpy as np
import pytest
import torch

from paper_2504_12984_amd import workloads as WL
from gpu_util import Prepared, assert_c_close, bits_of

pytestmark = pytest.mark.gpu

U = WL.KIND_UINT


def _cases():
    # streaming kernel with K over workgroups, tiled kernel with K over workgroups, then the
    # same two kinds again on smaller problems, then a call that needs no scratch at all
    return [WL.Case("noalloc_stream_big", 16, 8192, 2048, U, 4, group=128, zero="random", seed=9300),
            WL.Case("noalloc_tiled_big", 128, 8192, 2048, U, 4, group=128, act="bf16", scale_dtype="bf16",
                    zero="random", seed=9301),
            WL.Case("noalloc_stream_small", 5, 4096, 1024, U, 3, group=64, zero="random", seed=9302),
            WL.Case("noalloc_tiled_small", 100, 2048, 512, U, 6, group=128, act="bf16", scale_dtype="f16",
                    zero="random", seed=9303),
            WL.Case("noalloc_unsplit", 300, 512, 1024, U, 5, group=64, act="bf16", scale_dtype="bf16",
                    zero="random", seed=9304)]


def test_noalloc_matches_qgemm_on_calls_in_a_row_the_later_ones_smaller():
    from paper_2504_12984_amd import binding as B
    for k in range(4):
        B.qg_set_knob(k, 0)
    Ps = [Prepared(c) for c in _cases()]
    act = {"f16": B.QG_F16, "bf16": B.QG_BF16}
    plans = [B.qg_plan(P.wtype, P.case.group, P.case.M, P.case.N, P.case.K, act=act[P.case.act],
                       scale_dtype=act[P.case.scale_dtype]) for P in Ps]
    assert [p["splitk"] > 1 for p in plans] == [True, True, True, True, False], plans
    assert [p["path"] for p in plans] == [1, 2, 1, 2, 2], plans
    want = [P.gpu_c() for P in Ps]                           # the existing entry point
    refs = [P.oracle_c() for P in Ps]
    outs = [torch.empty_like(w) for w in want]
    for out in outs:
        out.zero_()                   # (torch loads its fill kernel on first use: before the measurement)
    # set-up call (M = 0, no pointers): the array's address on this device is looked up here
    t0 = Ps[0].wtype.c()
    assert B._lib.qgemm_noalloc(None, None, None, None, t0, 0, B.QG_F16, B.QG_F16, 128, 0, 64, 128, None, None) == B.QG_OK
    torch.cuda.synchronize()
    before = torch.cuda.mem_get_info()[0]
    # through the C entry point itself, back to back on one stream, twice over
    for rep in range(2):
        for P, out in zip(Ps, outs):
            out.zero_()
            c = P.case
            rc = B._lib.qgemm_noalloc(P.d_A.data_ptr(), P.d_packed.data_ptr(), P.d_scales.data_ptr(),
                                      P.d_zeros.data_ptr(), P.wtype.c(), 0, act[c.act], act[c.scale_dtype],
                                      c.group, c.M, c.N, c.K, out.data_ptr(), torch.cuda.current_stream().cuda_stream)
            assert rc == B.QG_OK, (c.name, rc, B._lib.qg_last_error())
        torch.cuda.synchronize()
        assert before - torch.cuda.mem_get_info()[0] < (1 << 20), "device memory in use grew across qgemm_noalloc calls"
        for P, out, w, ref in zip(Ps, outs, want, refs):
            assert_c_close(out, ref, f"{P.case.name} rep {rep}")
            assert np.array_equal(bits_of(out), bits_of(w)), f"{P.case.name} rep {rep}: bits differ from qgemm's"


def test_noalloc_and_qgemm_interleaved_keep_their_own_scratch():
    # the same split-K problem through both entry points alternately: each uses its own
    # arrival counters, so neither may disturb the other's
    from paper_2504_12984_amd import binding as B
    P = Prepared(_cases()[2])
    ref = P.oracle_c()
    first = P.gpu_c()
    out = torch.empty_like(first)
    for i in range(3):
        B.qgemm_noalloc(P.d_A, P.d_packed, P.d_scales, P.d_zeros, P.wtype, P.case.group, P.case.N, out)
        again = P.gpu_c()
        torch.cuda.synchronize()
        assert np.array_equal(bits_of(out), bits_of(first)) and np.array_equal(bits_of(again), bits_of(first)), i
    assert_c_close(out, ref, P.case.name)


def test_noalloc_refuses_a_request_beyond_its_scratch_and_says_so():
    from paper_2504_12984_amd import binding as B
    # forced split of K into 128 slabs: 128 slabs x 32 strips x 16 KiB of partial sums = 64 MiB
    case = WL.Case("noalloc_too_big", 64, 16384, 2048, U, 4, group=128, zero=8, seed=9310)
    P = Prepared(case)
    out = torch.empty((case.M, case.N), dtype=torch.float16, device="cuda")
    try:
        B.qg_set_knob(0, 1)
        B.qg_set_knob(1, 128)
        with pytest.raises(B.QgError) as err:
            B.qgemm_noalloc(P.d_A, P.d_packed, P.d_scales, P.d_zeros, P.wtype, case.group, case.N, out)
        assert err.value.status == B.QG_EUNSUPPORTED
        msg = B._lib.qg_last_error().decode()
        assert "qgemm_noalloc" in msg and "67108864" in msg and "33554432" in msg, msg
        assert_c_close(P.gpu_c(), P.oracle_c(), case.name + " through qgemm")      # qgemm takes a larger block
    finally:
        B.qg_set_knob(0, 0)
        B.qg_set_knob(1, 0)
    # and the fixed scratch still serves the automatic plan of the same problem
    B.qgemm_noalloc(P.d_A, P.d_packed, P.d_scales, P.d_zeros, P.wtype, case.group, case.N, out)
    assert_c_close(out, P.oracle_c(), case.name + " automatic")

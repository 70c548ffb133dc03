"""The C-ABI library loads and exports every symbol the headers under include/ declare.
No compute call is made here (runs without a GPU)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    inc = os.path.join(ROOT, "include")
    text = "\n".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    return sorted(set(re.findall(r"^QG_API\s+[\w\s\*]+?\b(\w+)\s*\(", text, flags=re.M)))


def test_header_declares_the_expected_entry_points():
    names = _declared()
    for must in ("qgemm", "qgemm_noalloc", "repack", "qdequant", "qgemm_packed_bytes", "qg_pack_codes", "qg_set_knob"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2504_12984_amd import binding as B
    lib = ctypes.CDLL(B.LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), name
    assert sorted(B.EXPORTS) == _declared()


def test_host_side_size_queries_and_status_strings():
    from paper_2504_12984_amd import binding as B
    assert B.qg_canonical_bytes(3, 8) == 3 and B.qg_canonical_bytes(5, 5) == 4
    assert B.qg_canonical_bytes(9, 8) == 0
    t = B.WType(B.QG_INT, 6)
    assert B.qgemm_packed_bytes(t, 128, 64) == 128 * 64 * 6 // 8      # BK*BN*6/8 bytes per tile
    assert B.qgemm_packed_bytes(t, 8192, 57344) == 8192 * 57344 * 6 // 8
    assert B.qgemm_packed_bytes(t, 100, 64) == 0 and B.qgemm_packed_bytes(t, 128, 65) == 0
    assert B.qgemm_packed_bytes(B.WType(B.QG_FLOAT, 6, 3, 2), 128, 64) == 6144
    assert B.qgemm_packed_bytes(B.WType(B.QG_FLOAT, 6, 3, 3), 128, 64) == 0   # 1+e+m != bits
    assert B._lib.qg_status_string(0) == b"ok"
    assert b"invalid" in B._lib.qg_status_string(-1)


def test_argument_errors_are_reported_before_anything_is_enqueued():
    from paper_2504_12984_amd import binding as B
    t = B.WType(B.QG_UINT, 4).c()
    # null pointers, bad shapes, bad bits: all rejected on the host
    assert B._lib.repack(None, t, 0, 128, 64, None, None) == B.QG_EINVAL
    assert B._lib.qgemm(None, None, None, None, t, 0, 0, 0, 128, 1, 64, 128, None, None) == B.QG_EINVAL
    assert B._lib.qgemm(None, None, None, None, t, 0, 0, 0, 128, 1, 64, 100, None, None) == B.QG_EINVAL
    assert B._lib.qgemm(None, None, None, None, B.WType(B.QG_UINT, 9).c(), 0, 0, 0, 128, 1, 64, 128, None, None) == B.QG_EINVAL
    assert B._lib.qdequant(None, None, None, t, 0, 0, 0, 96, 128, 64, None, None) == B.QG_EINVAL   # K % group
    assert B._lib.qdequant(None, None, None, t, 7, 0, 0, 128, 128, 64, None, None) == B.QG_EINVAL  # layout
    assert B._lib.qdequant(None, None, None, B.WType(B.QG_FLOAT, 8, 5, 2).c(), 0, 0, 0, 128, 128, 64, None, None) == B.QG_EUNSUPPORTED
    assert B._lib.qg_pack_codes(None, 0, 8, None, None) == B.QG_EINVAL
    assert B._lib.qg_pack_codes(None, 3, 0, None, None) == B.QG_OK


def test_codebook_and_int8_entry_points_reject_bad_arguments_on_the_host():
    from paper_2504_12984_amd import binding as B
    L = B._lib
    cb = B.WType(B.QG_CODEBOOK, 4).c()
    # codebook calls: bits out of range, null pointers, K % group, scale type combinations
    assert L.qgemm_codebook(None, None, None, None, 0, 0, 0, 128, 1, 64, 128, None, None) == B.QG_EINVAL
    assert L.qgemm_codebook(None, None, None, None, 9, 0, 0, 128, 1, 64, 128, None, None) == B.QG_EINVAL
    assert L.qgemm_codebook(None, None, None, None, 4, 0, 0, 128, 1, 64, 128, None, None) == B.QG_EINVAL      # null pointers
    assert L.qgemm_codebook(None, None, None, None, 4, 0, 0, 96, 1, 64, 128, None, None) == B.QG_EINVAL       # K % group
    assert L.qgemm_codebook(None, None, None, None, 4, 0, B.QG_BF16, 128, 1, 64, 128, None, None) == B.QG_EUNSUPPORTED
    assert L.qgemm_codebook(None, None, None, None, 4, 0, B.QG_E8M0, 32, 1, 64, 128, None, None) == B.QG_EUNSUPPORTED
    assert L.qgemm_codebook(None, None, None, None, 4, 0, 0, 128, 0, 64, 128, None, None) == B.QG_OK          # M = 0: nothing to do
    assert L.qdequant_codebook(None, None, None, 4, 0, 0, 128, 128, 64, None, None) == B.QG_EINVAL
    assert L.qdequant_codebook(None, None, None, 4, 0, 0, 128, 100, 64, None, None) == B.QG_EINVAL
    # the plain calls have no table: the codebook kind is an invalid argument there, and so is it for int8 activations
    assert L.qgemm(None, None, None, None, cb, 0, 0, 0, 128, 1, 64, 128, None, None) == B.QG_EINVAL
    assert L.qdequant(None, None, None, cb, 0, 0, 0, 128, 128, 64, None, None) == B.QG_EINVAL
    assert L.qgemm_a8(None, None, None, None, None, cb, 0, 0, 128, 1, 64, 128, None, None) == B.QG_EINVAL
    # repack takes the kind on the first layout only
    assert L.repack(None, cb, 1, 128, 64, None, None) == B.QG_EUNSUPPORTED
    assert L.repack(None, cb, 0, 128, 64, None, None) == B.QG_EINVAL                                          # null pointers
    assert B.qgemm_packed_bytes(B.WType(B.QG_CODEBOOK, 3), 128, 64) == 3072
    # int8 activations: float weights and group 32 have no kernel
    u4 = B.WType(B.QG_UINT, 4).c()
    assert L.qgemm_a8(None, None, None, None, None, B.WType(B.QG_FLOAT, 4, 2, 1).c(), 0, 0, 128, 1, 64, 128, None, None) == B.QG_EUNSUPPORTED
    assert L.qgemm_a8(None, None, None, None, None, u4, 0, 0, 32, 1, 64, 128, None, None) == B.QG_EUNSUPPORTED
    assert L.qgemm_a8(None, None, None, None, None, u4, 0, 0, 128, 1, 64, 128, None, None) == B.QG_EINVAL      # null pointers

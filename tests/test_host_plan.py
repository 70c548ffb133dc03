"""Host logic: which kernel, tile height, wavefront arrangement and split-K the
library picks for a shape (qg_plan: arithmetic only, runs without a GPU).
Checks the invariants the kernels rely on and the choices the measurements in
the design notes were taken with."""
import pytest

from paper_2504_12984_amd import binding as B

U4 = B.WType(B.QG_UINT, 4)
U3 = B.WType(B.QG_UINT, 3)
U8 = B.WType(B.QG_UINT, 8)


@pytest.fixture(autouse=True)
def _reset_knobs():
    yield
    for k in range(4):
        B.qg_set_knob(k, 0)


def test_small_m_streams_and_large_m_tiles():
    assert B.qg_plan(U4, 128, 1, 14336, 4096)["path"] == 1
    assert B.qg_plan(U4, 128, 32, 14336, 4096)["path"] == 1
    assert B.qg_plan(U4, 128, 65, 14336, 4096)["path"] == 2
    assert B.qg_plan(U4, 128, 4096, 57344, 8192) == {"path": 2, "variant": 0, "row_tile": 0, "splitk": 1,
                                                     "chunks_per_slab": 64}


def test_streaming_arrangements_of_the_named_workloads():
    # W3A16 decode: 224 strips, 32 chunks -> 16 wavefronts on one strip, no split
    p = B.qg_plan(U3, 128, 16, 14336, 4096)
    assert (p["variant"], p["splitk"]) == (12, 1)
    # signed sweep shape: 448 strips, long K -> two strips per workgroup, 16 wavefronts up to 6 bits, 8 above
    assert B.qg_plan(U4, 128, 16, 28672, 8192)["variant"] == 15
    assert B.qg_plan(U8, 128, 16, 28672, 8192)["variant"] == 14
    assert B.qg_plan(U4, 64, 16, 28672, 8192)["variant"] == 14      # two groups per chunk need the registers
    # type sweep shape: 896 strips -> four strips per workgroup
    assert B.qg_plan(U4, 128, 16, 57344, 8192)["variant"] == 16
    # K = N = 8192: 128 strips cannot fill 256 CUs -> K is split over workgroups
    p = B.qg_plan(U4, 128, 1, 8192, 8192)
    assert p["variant"] == 12 and p["splitk"] == 2 and p["chunks_per_slab"] == 32
    # short K: wavefronts per strip so that each keeps two chunks, 16 only for narrow codes on
    # enough strips, pairs of strips when there are many (measured: 16 wavefronts on 8-bit
    # codes or on 8-chunk strips cost 2-3x)
    assert B.qg_plan(U8, 128, 16, 14336, 4096)["variant"] == 10
    assert B.qg_plan(U8, 128, 16, 28672, 4096)["variant"] == 14
    assert B.qg_plan(U4, 128, 16, 28672, 4096)["variant"] == 15
    assert B.qg_plan(U4, 128, 16, 57344, 1024)["variant"] == 14
    assert B.qg_plan(U4, 128, 16, 57344, 2048)["variant"] == 16
    assert B.qg_plan(U4, 128, 16, 14336, 1024)["variant"] == 11
    p = B.qg_plan(U4, 128, 16, 4096, 4096)
    assert (p["variant"], p["splitk"]) == (10, 2)
    # long K on few strips: K in four even at under two chunks per wavefront, never deeper for it;
    # between 128 and 256 strips 8-wavefront workgroups (two share a CU) instead of 16
    p = B.qg_plan(U4, 128, 16, 4096, 14336)
    assert (p["variant"], p["splitk"]) == (12, 4)
    assert B.qg_plan(U8, 128, 16, 1024, 8192)["splitk"] == 4
    p = B.qg_plan(U4, 128, 16, 14336, 8192)
    assert (p["variant"], p["splitk"]) == (10, 2)
    assert B.qg_plan(U8, 128, 16, 14336, 8192)["variant"] == 14
    # several row tiles: pairs of strips whatever the length of K, no split on 192 strips or more
    assert B.qg_plan(U4, 128, 24, 28672, 4096)["variant"] == 26
    p = B.qg_plan(U4, 128, 24, 14336, 4096)
    assert (p["variant"], p["splitk"]) == (21, 1)
    # 17..32 and 33..64 rows: 2 and 4 row tiles per wavefront
    assert B.qg_plan(U4, 128, 32, 8192, 8192)["variant"] // 10 == 2
    assert B.qg_plan(U4, 128, 64, 8192, 8192)["variant"] // 10 == 4


@pytest.mark.parametrize("bits", [1, 4, 6, 8])
@pytest.mark.parametrize("K", [128, 384, 1024, 1408, 4096, 8192])
@pytest.mark.parametrize("N", [64, 2048, 8192, 14336, 57344])
@pytest.mark.parametrize("M", [65, 96, 128, 200, 256, 384, 512, 768, 1024, 4096])
def test_tiled_plan_invariants(M, N, K, bits):
    p = B.qg_plan(B.WType(B.QG_UINT, bits), 128, M, N, K)
    KC = K // 128
    assert p["path"] == 2 and p["row_tile"] in (0, 64, 128)
    sk, cps = p["splitk"], p["chunks_per_slab"]
    assert 1 <= sk <= 8 and sk * cps >= KC > (sk - 1) * cps          # slabs cover K, none is empty
    if sk > 1:
        assert p["row_tile"] in (64, 128)                            # 256-row tiles are never split
        assert cps % 2 == 0 and cps >= 4                             # whole pairs of chunks
        tiles = -(-M // p["row_tile"]) * -(-N // 256)
        assert tiles * sk <= 256                                     # one workgroup per CU at most
    if p["row_tile"] == 0:
        assert -(-M // 128) * -(-N // 256) > 128                     # big enough to fill the chip unsplit


def test_33_to_64_rows_take_the_tiled_kernel_on_all_but_small_problems():
    F6 = B.WType(B.QG_FLOAT, 6, 3, 2)
    for M in (33, 48, 64):
        # measured: tiled split-K faster (K = 8192, N = 28672: 57 against 71 us at 4 bits)
        for K, N, sk in ((8192, 28672, 2), (8192, 14336, 4), (28672, 8192, 8), (8192, 57344, 1), (1024, 57344, 1)):
            p = B.qg_plan(U4, 128, M, N, K)
            assert (p["path"], p["row_tile"], p["splitk"]) == (2, 64, sk), (M, K, N, p)
        # measured: streaming kernel faster or equal
        for K, N in ((8192, 8192), (4096, 4096), (14336, 4096), (2048, 8192), (128, 64)):
            assert B.qg_plan(U4, 128, M, N, K)["path"] == 1, (M, K, N)
        # float codes unpack more slowly in the tiled kernel: e3m2 stays on the streaming kernel
        assert B.qg_plan(F6, 128, M, 28672, 8192, act=B.QG_BF16)["path"] == 1
    for M in (1, 16, 32):
        assert B.qg_plan(U4, 128, M, 28672, 8192)["path"] == 1
    B.qg_set_knob(3, 41)                                   # a forced arrangement keeps the streaming kernel
    assert B.qg_plan(U4, 128, 64, 28672, 8192)["path"] == 1


def test_split_k_choices_of_the_measured_shapes():
    # K = N = 8192, 4-bit (the table in the design notes)
    got = {M: B.qg_plan(U4, 128, M, 8192, 8192) for M in (128, 256, 512)}
    assert (got[128]["row_tile"], got[128]["splitk"]) == (64, 4)
    assert (got[256]["row_tile"], got[256]["splitk"]) in ((64, 2), (128, 4))
    assert (got[512]["row_tile"], got[512]["splitk"]) == (128, 2)
    # short K: nothing to split
    assert B.qg_plan(U4, 128, 128, 8192, 1024)["splitk"] == 1


def test_knobs_force_the_plan_and_bad_arguments_are_rejected():
    B.qg_set_knob(0, 2); B.qg_set_knob(2, 128); B.qg_set_knob(1, 3)
    p = B.qg_plan(U4, 128, 40, 320, 1408)                            # 11 chunks in 3 slabs of 4
    assert (p["path"], p["row_tile"], p["splitk"], p["chunks_per_slab"]) == (2, 128, 3, 4)
    B.qg_set_knob(2, 256)
    assert B.qg_plan(U4, 128, 400, 320, 1408)["splitk"] == 1         # 256-row tiles are not split
    B.qg_set_knob(0, 1)
    with pytest.raises(Exception):
        B.qg_plan(U4, 128, 65, 320, 1408)                            # streaming kernel forced beyond 64 rows
    for k in range(4):
        B.qg_set_knob(k, 0)
    with pytest.raises(Exception):
        B.qg_plan(U4, 128, 16, 100, 1408)                            # N not a multiple of 64
    with pytest.raises(Exception):
        B.qg_plan(U4, 96, 16, 128, 1408)                             # group does not divide K
    assert B.qg_plan(U4, 128, 300, 512, 1024, layout=B.QG_LAYOUT_TILE128x64_R32)["path"] == 2
    assert B.qg_plan(U4, 0, 16, 128, 1408) == B.qg_plan(U4, 1408, 16, 128, 1408)    # 0 = one scale per column
    # group 32: 4-wavefront arrangements of the streaming kernel, tiled kernel beyond 64 rows
    assert B.qg_plan(U4, 32, 16, 28672, 8192)["variant"] == 11
    assert B.qg_plan(U4, 32, 300, 512, 1024)["path"] == 2
    with pytest.raises(Exception):
        B.qg_plan(U4, 32, 300, 512, 1024, layout=B.QG_LAYOUT_TILE128x64_R32)
    with pytest.raises(Exception):
        B.qg_plan(U4, 16, 16, 512, 1024)


def test_forced_arrangement_must_cover_the_rows():
    # an arrangement with one row tile cannot serve 64 rows (rows 16..63 would stay unwritten)
    B.qg_set_knob(3, 11)
    assert B.qg_plan(U4, 128, 16, 512, 1408)["variant"] == 11
    with pytest.raises(B.QgError) as e:
        B.qg_plan(U4, 128, 64, 512, 1408)
    assert e.value.status == B.QG_EINVAL
    B.qg_set_knob(3, 46)
    assert B.qg_plan(U4, 128, 64, 512, 1408)["variant"] == 46
    with pytest.raises(B.QgError):
        B.qg_plan(U4, 128, 20, 512, 1408)
    # over blocks of 64 rows every block is checked: 64 + 6 rows need 4 row tiles, then 1
    B.qg_set_knob(0, 3)
    with pytest.raises(B.QgError):
        B.qg_plan(U4, 128, 70, 512, 1408)
    assert B.qg_plan(U4, 128, 128, 512, 1408)["variant"] == 46


def test_tiled_kernels_take_operands_below_two_gib_only():
    # A = M x K x 2 bytes: 2^31 at M = 131072, K = 8192
    assert B.qg_plan(U4, 128, 131071, 256, 8192)["path"] == 2
    for layout in (0, 1):
        with pytest.raises(B.QgError) as e:
            B.qg_plan(U4, 128, 131072, 256, 8192, layout=layout)
        assert e.value.status == B.QG_EUNSUPPORTED
    # packed weight = K x N x bits / 8: 2^31 at 8 bits, K = 32768, N = 65536; 7 bits fit
    with pytest.raises(B.QgError):
        B.qg_plan(U8, 128, 100, 65536, 32768)
    assert B.qg_plan(B.WType(B.QG_UINT, 7), 128, 100, 65536, 32768)["path"] == 2
    # the streaming kernel addresses with 64-bit pointers and takes them all
    assert B.qg_plan(U8, 128, 16, 65536, 32768)["path"] == 1


def test_batch_size_axis_of_the_paper():
    # K = 8192, N = 57344 (the type-sweep shape) at the paper's batch sizes
    F6 = B.WType(B.QG_FLOAT, 6, 3, 2)
    for t in (U4, F6):
        for M in (1, 4, 8, 16):
            p = B.qg_plan(t, 128, M, 57344, 8192)
            assert (p["path"], p["variant"], p["splitk"]) == (1, 16, 1), (M, p)      # 896 strips: four per workgroup
        for M in (4096, 8192, 12288):
            p = B.qg_plan(t, 128, M, 57344, 8192)
            # whole rounds of 256-row tiles, the rest in a second launch; never split
            assert p == {"path": 2, "variant": 0, "row_tile": 0, "splitk": 1, "chunks_per_slab": 64}, (M, p)


def test_block_scaled_weights_plan_and_refusals():
    F4, F8, F6 = B.WType(B.QG_FLOAT, 4, 2, 1), B.WType(B.QG_FLOAT, 8, 4, 3), B.WType(B.QG_FLOAT, 6, 3, 2)
    E8 = B.QG_E8M0
    # streaming kernel (every arrangement is open to them) and tiled kernel like any other weight
    assert B.qg_plan(F4, 32, 1, 57344, 8192, act=B.QG_BF16, scale_dtype=E8)["variant"] == 16
    assert B.qg_plan(F8, 32, 16, 8192, 8192, act=B.QG_F16, scale_dtype=E8)["path"] == 1
    assert B.qg_plan(F8, 32, 4096, 8192, 8192, act=B.QG_BF16, scale_dtype=E8)["path"] == 2
    # the same weights with 16-bit scales and group 32 keep to the four-wavefront arrangements
    assert B.qg_plan(F4, 32, 1, 57344, 8192, act=B.QG_BF16, scale_dtype=B.QG_F16)["variant"] == 11
    for t, group, layout in ((F6, 32, 0), (U4, 32, 0), (F4, 128, 0), (F4, 32, 1)):
        with pytest.raises(B.QgError) as e:
            B.qg_plan(t, group, 16, 8192, 8192, act=B.QG_BF16, scale_dtype=E8, layout=layout)
        assert e.value.status == B.QG_EUNSUPPORTED, (t, group, layout)
    B.qg_set_knob(0, 4)
    with pytest.raises(B.QgError) as e:
        B.qg_plan(F4, 32, 16, 8192, 8192, act=B.QG_BF16, scale_dtype=E8)
    assert e.value.status == B.QG_EUNSUPPORTED


def test_dequantise_first_path_plan():
    B.qg_set_knob(0, 4)
    p = B.qg_plan(U4, 128, 4096, 57344, 8192, act=B.QG_BF16)
    assert (p["path"], p["splitk"]) == (4, 1)
    assert B.qg_plan(U4, 128, 128, 2048, 8192, act=B.QG_BF16)["splitk"] > 1      # the same tile / split choices as the tiled kernel
    with pytest.raises(B.QgError) as e:                                            # K*N*2 bytes must stay below 2 GiB
        B.qg_plan(U4, 128, 128, 65536, 16384, act=B.QG_BF16)
    assert e.value.status == B.QG_EUNSUPPORTED


def test_codebook_weights_plan_like_the_integer_type_and_refusals():
    CB4, CB8 = B.WType(B.QG_CODEBOOK, 4), B.WType(B.QG_CODEBOOK, 8)
    for M, N, K in ((1, 57344, 8192), (16, 8192, 8192), (48, 28672, 8192), (300, 8192, 4096), (4096, 57344, 8192)):
        assert B.qg_plan(CB4, 128, M, N, K) == B.qg_plan(U4, 128, M, N, K), (M, N, K)
        if M < 1024:
            assert B.qg_plan(CB8, 64, M, N, K, act=B.QG_BF16) == B.qg_plan(U8, 64, M, N, K, act=B.QG_BF16), (M, N, K)
    # wide codebooks on many rows: de-quantise first (the paper's prefill variant), while its buffer stays below 2 GiB
    assert B.qg_plan(CB8, 128, 1024, 57344, 8192)["path"] == 4
    assert B.qg_plan(B.WType(B.QG_CODEBOOK, 5), 128, 4096, 8192, 8192)["path"] == 4
    assert B.qg_plan(CB8, 128, 1023, 57344, 8192)["path"] == 2
    assert B.qg_plan(CB8, 128, 4096, 65536, 16384)["path"] == 2
    assert B.qg_plan(CB4, 128, 4096, 57344, 8192)["path"] == 2
    B.qg_set_knob(0, 2)
    assert B.qg_plan(CB8, 128, 4096, 57344, 8192)["path"] == 2
    B.qg_set_knob(0, 0)
    # only the first layout has lookup kernels; block scales do not combine with a table
    assert B.qgemm_packed_bytes(CB4, 256, 128) == 256 * 128 // 2
    assert B.qgemm_packed_bytes(CB4, 256, 128, layout=B.QG_LAYOUT_TILE128x64_R32) == 0
    with pytest.raises(B.QgError) as e:
        B.qg_plan(CB4, 128, 16, 8192, 8192, layout=B.QG_LAYOUT_TILE128x64_R32)
    assert e.value.status == B.QG_EUNSUPPORTED
    with pytest.raises(B.QgError) as e:
        B.qg_plan(CB4, 32, 16, 8192, 8192, act=B.QG_BF16, scale_dtype=B.QG_E8M0)
    assert e.value.status == B.QG_EUNSUPPORTED
    for bad in (B.WType(B.QG_CODEBOOK, 0), B.WType(B.QG_CODEBOOK, 9), B.WType(B.QG_CODEBOOK, 4, 1, 2)):
        with pytest.raises(B.QgError) as e:
            B.qg_plan(bad, 128, 16, 8192, 8192)
        assert e.value.status == B.QG_EINVAL


def test_matrix_vector_path_plan():
    B.qg_set_knob(0, 5)
    p = B.qg_plan(U3, 128, 1, 14336, 4096)
    assert (p["path"], p["variant"]) == (5, 16) and p["splitk"] == 1        # 32 chunks, 16 wavefronts, 224 strips: K in one piece
    assert B.qg_plan(U3, 128, 4, 14336, 4096)["variant"] == 8               # several rows: the ring of 16 wavefronts would spill
    assert B.qg_plan(U8, 128, 1, 8192, 8192)["variant"] == 8
    assert B.qg_plan(U4, 128, 1, 512, 512)["variant"] == 4
    p = B.qg_plan(U4, 128, 1, 8192, 8192)
    assert p["variant"] == 16 and p["splitk"] == 2 and p["chunks_per_slab"] == 32
    B.qg_set_knob(3, 8)
    assert B.qg_plan(U4, 128, 1, 8192, 8192)["variant"] == 8
    B.qg_set_knob(3, 0)
    with pytest.raises(B.QgError) as e:
        B.qg_plan(U4, 128, 5, 8192, 8192)
    assert e.value.status == B.QG_EINVAL

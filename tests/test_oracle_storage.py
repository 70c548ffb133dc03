"""Pins for the oracle's compact storage (paper: Section "Storage of
Low-Precision Data").  Nothing here calls the HIP path."""
import numpy as np
import pytest

from oracle import qgemm_oracle as O
from conftest import read_golden


def _hex(xs):
    return np.array([int(x, 16) for x in xs], dtype=np.uint8)


@pytest.mark.parametrize("tag,bits", [("u3", 3), ("i6", 6), ("u5", 5)])
def test_hand_derived_streams(tag, bits):
    g = read_golden("bitstreams.txt")
    codes = np.array([int(x) for x in g[f"{tag}_codes"]], dtype=np.uint8)
    want = _hex(g[f"{tag}_bytes"])
    got = O.pack_canonical(codes, bits)
    assert got.tolist() == want.tolist()
    assert O.unpack_canonical(want, bits, codes.size).tolist() == codes.tolist()


def test_i6_patterns_are_twos_complement_of_golden_values():
    g = read_golden("bitstreams.txt")
    vals = [int(x) for x in g["i6_values"]]
    codes = [int(x) for x in g["i6_codes"]]
    tab = O.code_values(O.KIND_INT, 6)
    assert [tab[c] for c in codes] == vals


@pytest.mark.parametrize("bits", range(1, 9))
def test_bit_by_bit_definition(bits):
    """Stream bit j == bit (j % b) of code j // b, checked with Python loops."""
    rng = np.random.default_rng(bits)
    codes = rng.integers(0, 1 << bits, size=77, dtype=np.uint8)
    buf = O.pack_canonical(codes, bits)
    assert buf.size == (77 * bits + 7) // 8
    for j in range(buf.size * 8):
        got = (int(buf[j // 8]) >> (j % 8)) & 1
        e = j // bits
        want = (int(codes[e]) >> (j % bits)) & 1 if e < codes.size else 0
        assert got == want, (bits, j)


def test_one_bit_equals_numpy_packbits():
    rng = np.random.default_rng(1)
    codes = rng.integers(0, 2, size=1003, dtype=np.uint8)
    assert O.pack_canonical(codes, 1).tolist() == np.packbits(codes, bitorder="little").tolist()
    assert O.unpack_canonical(np.packbits(codes, bitorder="little"), 1, 1003).tolist() == codes.tolist()


def test_byte_and_nibble_identities():
    rng = np.random.default_rng(2)
    c8 = rng.integers(0, 256, size=300, dtype=np.uint8)
    assert O.pack_canonical(c8, 8).tolist() == c8.tolist()
    c4 = rng.integers(0, 16, size=300, dtype=np.uint8)
    assert O.pack_canonical(c4, 4).tolist() == (c4[0::2] | (c4[1::2] << 4)).tolist()
    c2 = rng.integers(0, 4, size=400, dtype=np.uint8)
    want2 = c2[0::4] | (c2[1::4] << 2) | (c2[2::4] << 4) | (c2[3::4] << 6)
    assert O.pack_canonical(c2, 2).tolist() == want2.tolist()


@pytest.mark.parametrize("bits", range(1, 9))
@pytest.mark.parametrize("count", [1, 7, 8, 9, 64, 1001])
def test_round_trip_random_and_adversarial(bits, count):
    rng = np.random.default_rng(100 * bits + count)
    top = (1 << bits) - 1
    pats = [
        rng.integers(0, top + 1, size=count, dtype=np.uint8),
        np.full(count, top, dtype=np.uint8),
        np.zeros(count, dtype=np.uint8),
        (np.arange(count) % 2 * top).astype(np.uint8),
        ((np.arange(count) == count // 2) * 1).astype(np.uint8),
        (np.arange(count) % (top + 1)).astype(np.uint8),
    ]
    for codes in pats:
        buf = O.pack_canonical(codes, bits)
        assert buf.size == O.packed_nbytes(count, bits) == -(-count * bits // 8)
        assert O.unpack_canonical(buf, bits, count).tolist() == codes.tolist()
        # pad bits are zero
        total = int(np.unpackbits(buf, bitorder="little").sum())
        assert total == sum(bin(int(c)).count("1") for c in codes)


def test_single_set_bit_moves_to_the_right_place():
    for bits in range(1, 9):
        for e in range(20):
            for b in range(bits):
                codes = np.zeros(20, dtype=np.uint8)
                codes[e] = 1 << b
                buf = O.pack_canonical(codes, bits)
                j = e * bits + b
                want = np.zeros_like(buf)
                want[j // 8] = 1 << (j % 8)
                assert buf.tolist() == want.tolist()


def test_unpack_elements_gathers_arbitrary_indices():
    rng = np.random.default_rng(5)
    for bits in range(1, 9):
        codes = rng.integers(0, 1 << bits, size=(37, 53), dtype=np.uint8)
        buf = O.pack_canonical(codes, bits)
        idx = rng.integers(0, codes.size, size=(11, 13))
        assert O.unpack_elements(buf, bits, idx).tolist() == codes.reshape(-1)[idx].tolist()


def test_tile_byte_count_identity_of_the_paper():
    # an i6 [BK, BN] tile is BK*BN*6/8 bytes; 32 threads x 4 i6 = 32 x 3 bytes
    for BK, BN in [(16, 8), (32, 64), (128, 64)]:
        assert O.packed_nbytes(BK * BN, 6) == BK * BN * 6 // 8
    assert O.packed_nbytes(4, 6) == 3

"""CPU oracle for the mixed-precision matmul  C[M,N] = A[M,K] . dequant(W[K,N]).

THIS IS TEST INFRASTRUCTURE.  It is a plain, slow, fp64 NumPy statement of what
the GPU library must compute.  It shares no code with the HIP path, imports
nothing from the product package, and must only be imported by the tests, by
the smoke check and by the benchmark's cpu_baseline leg.

What follows the paper and what is a reading of it
--------------------------------------------------
* The contraction C = A x B with A in a 16-bit float type and B in a low-bit
  type is the paper's problem statement (Section "An Example of Tilus Program").
* Compact storage -- sub-byte values packed without bit gaps into a byte
  array, a value possibly spanning two bytes, loaded with AND / SHIFT / OR and
  stored with mask-clear + OR -- is Section "Storage of Low-Precision Data".
  The paper's figure that fixes the bit order is not available; the reading
  used here is little-endian: element e occupies stream bits [e*b, (e+1)*b),
  stream bit j is bit (j mod 8) of byte (j div 8), low code bits first.
* The type families (uint1..8, int2..8, float3..8 with any exponent/mantissa
  split) are listed in Section "Key Ideas".  The paper gives no encoding
  details; the readings used here are: intk is two's complement in k bits
  (int1 = {0, -1}); floatk is sign | exponent | mantissa with bias
  2^(e-1)-1, gradual underflow, no infinities, and no NaNs except the two
  all-ones-magnitude codes of e4m3 (the usual "fn" 8-bit float).
* De-quantisation ("casting and de-quantizing to float16", Section "Efficient
  Low-Precision Support in LLMs") is not given a formula in the paper.  The
  reading used here is the standard affine group form
        w = (value(code) - z[k // g, n]) * s[k // g, n]
  evaluated exactly, then rounded ONCE, round-to-nearest-even, to the
  activation type; the contraction then runs over the rounded weights, which
  is what feeding a cast tile to a matrix instruction means.

* int8 activations (named as supported in Section "Arbitrary Data Type Support", nothing
  more is said): integer weights only, the sum over the rows of one scale group is an exact
  integer, the weight scale multiplies that sum, a per-row fp32 activation scale multiplies
  the row (qgemm_int8).

* Codebook quantisation (named in the closing section as something a lookup instruction
  would add, with no formula): the reading used here is one table of 2^k half-precision
  levels per weight matrix, w = table[code] * s[k // g, n], rounded once to the activation
  type; no zero-point (codebook_exact, qgemm_codebook_from_stream).

Parity pins (tests/test_oracle_*.py): hand-derived bit streams, numpy.packbits
for 1-bit, nibble/byte identities for 4/8-bit, exact-rational evaluation of the
float formats, torch's float8_e4m3fn table, numpy/torch half and bfloat16 casts,
integer matmul for uint8 weights, one-hot rows, brute-force triple loops; for the int8
leg: numpy int64 matmul, exact-rational triple loops, agreement with the 16-bit-activation
contraction wherever that one is exact, the row-sum form of the zero-point; for the codebook
leg: tables that reproduce the integer and float types (value tables of uintk - z, e2m1,
e4m3), exact-rational loops, one-hot rows, permuted tables.
The paper prints no numeric tensor example, so beyond those pins parity with
the paper's own implementation is unpinned.
"""
from __future__ import annotations

import numpy as np

KIND_UINT, KIND_INT, KIND_FLOAT = 0, 1, 2


# --------------------------------------------------------------------------
# Compact storage (Section "Storage of Low-Precision Data")
# --------------------------------------------------------------------------
def packed_nbytes(count: int, bits: int) -> int:
    """Bytes needed for `count` codes of `bits` bits with no gaps."""
    return (count * bits + 7) // 8


def pack_canonical(codes: np.ndarray, bits: int) -> np.ndarray:
    """Store codes (flattened, row-major) into the canonical byte stream.

    Store rule of the paper: clear the target bits, OR the value in; a value
    may touch two consecutive bytes.  The buffer starts zeroed so the clear is
    a no-op; each element contributes (code << shift) to byte i and, if it
    crosses the byte boundary, (code >> (8 - shift)) to byte i + 1.
    """
    assert 1 <= bits <= 8
    c = np.ascontiguousarray(codes, dtype=np.uint8).reshape(-1)
    assert not np.any(c >> bits) if bits < 8 else True, "code wider than bits"
    count = c.size
    out = np.zeros(packed_nbytes(count, bits) + 1, dtype=np.uint8)
    # Eight consecutive elements always occupy exactly `bits` whole bytes, so
    # the (shift, byte) pattern repeats with period 8; walk the 8 phases.
    for phase in range(8):
        sel = c[phase::8].astype(np.uint16)
        if sel.size == 0:
            continue
        bit0 = phase * bits
        byte0, shift = bit0 >> 3, bit0 & 7
        idx = byte0 + bits * np.arange(sel.size, dtype=np.int64)
        word = sel << shift                      # up to 15 significant bits
        out[idx] |= (word & 0xFF).astype(np.uint8)
        if shift + bits > 8:
            out[idx + 1] |= (word >> 8).astype(np.uint8)
    return out[:-1]


def unpack_elements(buf: np.ndarray, bits: int, elem_idx: np.ndarray) -> np.ndarray:
    """Load the codes at flat element indices `elem_idx` from the stream.

    Load rule of the paper: AND out the relevant bits of each touched byte,
    SHIFT them into place, OR the (at most two) parts together.
    """
    assert 1 <= bits <= 8
    b = np.asarray(buf, dtype=np.uint8).reshape(-1)
    e = np.asarray(elem_idx, dtype=np.int64)
    bit0 = e * bits
    i, shift = bit0 >> 3, (bit0 & 7).astype(np.uint16)
    lo = b[i].astype(np.uint16)
    nxt = np.minimum(i + 1, b.size - 1)
    hi = np.where(shift + bits > 8, b[nxt].astype(np.uint16), 0)
    word = lo | (hi << 8)
    return ((word >> shift) & ((1 << bits) - 1)).astype(np.uint8)


def unpack_canonical(buf: np.ndarray, bits: int, count: int) -> np.ndarray:
    """All `count` codes of the stream, in element order."""
    out = np.empty(count, dtype=np.uint8)
    step = 1 << 22
    for s in range(0, count, step):
        t = min(count, s + step)
        out[s:t] = unpack_elements(buf, bits, np.arange(s, t, dtype=np.int64))
    return out


# --------------------------------------------------------------------------
# Code -> value (type families of Section "Key Ideas")
# --------------------------------------------------------------------------
def code_values(kind: int, bits: int, ebits: int = 0, mbits: int = 0) -> np.ndarray:
    """fp64 value of every one of the 2^bits codes (NaN where not finite)."""
    n = 1 << bits
    c = np.arange(n, dtype=np.int64)
    if kind == KIND_UINT:
        return c.astype(np.float64)
    if kind == KIND_INT:
        return np.where(c >= n // 2, c - n, c).astype(np.float64)
    if kind == KIND_FLOAT:
        assert 1 + ebits + mbits == bits and ebits >= 1 and mbits >= 0
        bias = (1 << (ebits - 1)) - 1
        sign = (c >> (bits - 1)) & 1
        E = (c >> mbits) & ((1 << ebits) - 1)
        Mn = c & ((1 << mbits) - 1)
        frac = Mn.astype(np.float64) / float(1 << mbits)
        sub = np.ldexp(frac, 1 - bias)                         # E == 0
        nor = np.ldexp(1.0 + frac, (E - bias).astype(np.int64))  # E > 0
        v = np.where(E == 0, sub, nor)
        v = np.where(sign == 1, -v, v)                         # keeps -0.0
        if (ebits, mbits) == (4, 3):                           # e4m3 "fn"
            v = np.where((E == 15) & (Mn == 7), np.nan, v)
        return v
    raise ValueError("unknown kind")


def finite_codes(kind: int, bits: int, ebits: int = 0, mbits: int = 0) -> np.ndarray:
    """The codes whose value is finite, ascending."""
    v = code_values(kind, bits, ebits, mbits)
    return np.nonzero(np.isfinite(v))[0].astype(np.uint8)


# --------------------------------------------------------------------------
# One rounding, round-to-nearest-even, to the activation type
# --------------------------------------------------------------------------
_FMT = {"f16": (5, 10), "bf16": (8, 7)}


def round_rne(x: np.ndarray, fmt: str) -> np.ndarray:
    """Round fp64 values to a binary float format (returned still as fp64).

    x = f * 2^e with f in [0.5, 1).  The spacing of the target format around x
    is 2^(max(e - 1, emin) - mbits); dividing by it is exact in fp64, rint is
    round-half-to-even, multiplying back is exact.  Gradual underflow is kept;
    magnitudes that round above the largest finite value become infinite.
    """
    ebits, mbits = _FMT[fmt]
    bias = (1 << (ebits - 1)) - 1
    emin = 1 - bias
    x = np.asarray(x, dtype=np.float64)
    _, e = np.frexp(x)
    q_exp = np.maximum(e.astype(np.int64) - 1, emin) - mbits
    y = np.ldexp(np.rint(np.ldexp(x, -q_exp)), q_exp)
    max_finite = (2.0 - 2.0 ** (-mbits)) * 2.0 ** bias
    y = np.where(np.abs(y) > max_finite, np.copysign(np.inf, x), y)
    return np.where(np.isfinite(x), y, x)


def to_bits(y: np.ndarray, fmt: str) -> np.ndarray:
    """uint16 bit pattern of values already representable in `fmt`."""
    y = np.asarray(y, dtype=np.float64)
    if fmt == "f16":
        return y.astype(np.float16).view(np.uint16)
    if fmt == "bf16":
        return (y.astype(np.float32).view(np.uint32) >> 16).astype(np.uint16)
    raise ValueError(fmt)


def from_bits(u: np.ndarray, fmt: str) -> np.ndarray:
    """fp64 value of uint16 bit patterns of `fmt` (exact widening)."""
    u = np.asarray(u, dtype=np.uint16)
    if fmt == "f16":
        return u.view(np.float16).astype(np.float64)
    if fmt == "bf16":
        return (u.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    raise ValueError(fmt)


# --------------------------------------------------------------------------
# Power-of-two block scales (microscaling; the paper's closing remark that
# microscaling types are "a more fine-grained quantization" it could support)
# --------------------------------------------------------------------------
def e8m0_values(e: np.ndarray) -> np.ndarray:
    """fp64 value of 8-bit exponent-only scales: 2^(e - 127); the code 255 is NaN.

    This is the shared-scale format of the OCP microscaling types (one scale per
    block of 32 elements).  With such scales the de-quantised weight
    value(code) * 2^(e - 127) needs no rounding while it stays inside the target
    format's range, so the rest of the oracle (dequant_exact, round_rne) applies
    unchanged with these values as `scales`.
    """
    e = np.asarray(e, dtype=np.uint8).astype(np.int64)
    return np.where(e == 255, np.nan, np.ldexp(1.0, e - 127))


# --------------------------------------------------------------------------
# De-quantise and contract
# --------------------------------------------------------------------------
def dequant_exact(codes, kind, bits, ebits, mbits, scales, zeros, group):
    """w = (value(code) - z) * s in fp64, unrounded.

    codes  [K, N]  uint8 bit patterns
    scales [K/group, N] fp64 (the 16-bit scales widened exactly)
    zeros  [K/group, N] integers in the code-value domain, or None for 0
    """
    codes = np.asarray(codes)
    K, N = codes.shape
    assert K % group == 0
    v = code_values(kind, bits, ebits, mbits)[codes]           # [K, N] fp64
    gi = np.arange(K) // group
    s = np.asarray(scales, dtype=np.float64)[gi]               # [K, N]
    if zeros is not None:
        v = v - np.asarray(zeros).astype(np.float64)[gi]
    return v * s


def dequant_rounded(codes, kind, bits, ebits, mbits, scales, zeros, group, act):
    """The rounded weights W^ = rne_act(w) as fp64, plus their bit patterns."""
    w = dequant_exact(codes, kind, bits, ebits, mbits, scales, zeros, group)
    wr = round_rne(w, act)
    return wr, to_bits(wr, act)


def gemm_fp64(A: np.ndarray, W: np.ndarray) -> np.ndarray:
    """C = A . W in fp64."""
    return np.asarray(A, dtype=np.float64) @ np.asarray(W, dtype=np.float64)


def qgemm_from_stream(A, stream, kind, bits, ebits, mbits, scales, zeros, group,
                      K, N, act, cols=None, col_block=1024):
    """End to end from the canonical byte stream: unpack, de-quantise, round,
    contract.  `cols` restricts the result to the given output columns (each
    column of C depends on one column of W only).  Returns C_ref fp64 [M, len].
    """
    A = np.asarray(A, dtype=np.float64)
    cols = np.arange(N, dtype=np.int64) if cols is None else np.asarray(cols, dtype=np.int64)
    scales = np.asarray(scales, dtype=np.float64)
    out = np.empty((A.shape[0], cols.size), dtype=np.float64)
    rows = np.arange(K, dtype=np.int64)[:, None] * N
    for s in range(0, cols.size, col_block):
        cb = cols[s:s + col_block]
        codes = unpack_elements(stream, bits, rows + cb[None, :])
        z = None if zeros is None else np.asarray(zeros)[:, cb]
        wr, _ = dequant_rounded(codes, kind, bits, ebits, mbits, scales[:, cb], z, group, act)
        out[:, s:s + cb.size] = gemm_fp64(A, wr)
    return out


# --------------------------------------------------------------------------
# int8 activations (Section "Arbitrary Data Type Support": operand A may be an
# 8-bit type; the paper names int8 beside float16 and bfloat16)
# --------------------------------------------------------------------------
def int_weights(codes, kind, bits, zeros, group):
    """value(code) - z as exact integers (int64) [K, N]; integer weight kinds only."""
    if kind not in (KIND_UINT, KIND_INT):
        raise ValueError("int8 activations multiply integer weights (uintk / intk) only")
    codes = np.asarray(codes)
    K, N = codes.shape
    assert K % group == 0
    v = code_values(kind, bits)[codes].astype(np.int64)
    if zeros is not None:
        v = v - np.asarray(zeros).astype(np.int64)[np.arange(K) // group]
    return v


def qgemm_int8(A8, a_scale, codes, kind, bits, scales, zeros, group):
    """C[m,n] = a_scale[m] * sum_g s[g,n] * ( sum_{k in group g} A8[m,k] * (value(code[k,n]) - z[g,n]) ).

    The paper says that int8 is a supported activation type and gives nothing more; this is
    the reading used here.  An integer matrix instruction can only multiply integers, so the
    inner sum over the rows of one scale group is an exact integer, the group's weight scale
    (a 16-bit float widened exactly) multiplies that sum, the groups are added, and a
    per-row activation scale (fp32, the usual per-token quantisation of activations; None =
    1) multiplies the row.  Evaluated here in fp64 after the exact integer part; the result
    is NOT rounded to the output type (the comparison tolerance covers that rounding).

    The integer inner sums are formed with a float64 matrix product of integer-valued
    operands: every product is below 2^15 and every sum below 2^15 * K, far below 2^53,
    so each float64 operation is exact whatever order the library adds in.

    A8 [M, K] int8; a_scale [M] or None; codes [K, N] uint8 patterns; scales [K/group, N]
    fp64; zeros [K/group, N] integers or None.  Returns fp64 [M, N].
    """
    A8 = np.asarray(A8)
    assert A8.dtype == np.int8
    w = int_weights(codes, kind, bits, zeros, group)
    K, N = w.shape
    Af, wf = A8.astype(np.float64), w.astype(np.float64)
    s = np.asarray(scales, dtype=np.float64)
    C = np.zeros((A8.shape[0], N), dtype=np.float64)
    for g in range(K // group):
        rows = slice(g * group, (g + 1) * group)
        C += (Af[:, rows] @ wf[rows]) * s[g][None, :]
    if a_scale is not None:
        C *= np.asarray(a_scale, dtype=np.float64)[:, None]
    return C


def qgemm_int8_from_stream(A8, a_scale, stream, kind, bits, scales, zeros, group, K, N, cols=None, col_block=1024):
    """qgemm_int8 from the canonical byte stream, optionally on a subset of output columns."""
    cols = np.arange(N, dtype=np.int64) if cols is None else np.asarray(cols, dtype=np.int64)
    scales = np.asarray(scales, dtype=np.float64)
    out = np.empty((np.asarray(A8).shape[0], cols.size), dtype=np.float64)
    rows = np.arange(K, dtype=np.int64)[:, None] * N
    for s0 in range(0, cols.size, col_block):
        cb = cols[s0:s0 + col_block]
        codes = unpack_elements(stream, bits, rows + cb[None, :])
        z = None if zeros is None else np.asarray(zeros)[:, cb]
        out[:, s0:s0 + cb.size] = qgemm_int8(A8, a_scale, codes, kind, bits, scales[:, cb], z, group)
    return out


# --------------------------------------------------------------------------
# Codebook quantisation (the paper's closing section: codebook schemes such as
# LCQ would be served by adding a lookup instruction)
# --------------------------------------------------------------------------
def codebook_exact(codes, table, scales, group):
    """w = table[code] * s in fp64, unrounded.

    The paper says only that a lookup instruction would accommodate codebook quantisation;
    this is the reading used here.  A k-bit code is an index into ONE table of 2^k levels
    per weight matrix (LCQ learns one companding function, hence one set of levels, per
    layer); the levels are half-precision numbers whatever the activation type; the
    group scale multiplies the level as it multiplies value(code) - z in the affine form;
    there is no zero-point (a table can hold any offset).

    codes  [K, N]  uint8 indices below len(table)
    table  [2^k]   fp64 (half-precision levels widened exactly)
    scales [K/group, N] fp64
    """
    codes = np.asarray(codes)
    table = np.asarray(table, dtype=np.float64)
    K, N = codes.shape
    assert K % group == 0 and table.ndim == 1
    assert int(codes.max(initial=0)) < table.size
    gi = np.arange(K) // group
    return table[codes] * np.asarray(scales, dtype=np.float64)[gi]


def codebook_rounded(codes, table, scales, group, act):
    """The rounded weights rne_act(table[code] * s) as fp64, plus their bit patterns."""
    wr = round_rne(codebook_exact(codes, table, scales, group), act)
    return wr, to_bits(wr, act)


def qgemm_codebook_from_stream(A, stream, bits, table, scales, group, K, N, act, cols=None, col_block=1024):
    """C = A . rne_act(table[code] * s) from the canonical byte stream, optionally on a
    subset of output columns.  Returns fp64 [M, len(cols)]."""
    A = np.asarray(A, dtype=np.float64)
    cols = np.arange(N, dtype=np.int64) if cols is None else np.asarray(cols, dtype=np.int64)
    scales = np.asarray(scales, dtype=np.float64)
    out = np.empty((A.shape[0], cols.size), dtype=np.float64)
    rows = np.arange(K, dtype=np.int64)[:, None] * N
    for s0 in range(0, cols.size, col_block):
        cb = cols[s0:s0 + col_block]
        codes = unpack_elements(stream, bits, rows + cb[None, :])
        wr, _ = codebook_rounded(codes, table, scales[:, cb], group, act)
        out[:, s0:s0 + cb.size] = gemm_fp64(A, wr)
    return out


def within_tolerance(C, C_ref, atol=1e-2, rtol=5e-3) -> np.ndarray:
    """Elementwise  |C - C_ref| <= atol + rtol * |C_ref|."""
    C = np.asarray(C, dtype=np.float64)
    return np.abs(C - C_ref) <= atol + rtol * np.abs(C_ref)

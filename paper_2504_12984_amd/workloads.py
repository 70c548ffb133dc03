"""Seeded synthetic inputs for the quantised-matmul workloads.

This module only draws numbers.  It holds none of the method's arithmetic (no
packing, no de-quantisation, no layout knowledge) and imports neither the HIP
binding nor the CPU oracle, so both sides can be fed the same bits from it.

The paper benchmarks matmul shapes taken from LLM layers with dummy weights and
inputs (Section "Performance of Low-Precision Kernels", artifact appendix "Data
sets"); the cases below are dense i.i.d. stand-ins of those shapes.

Draw order per case, from numpy Generator(PCG64(seed)):  A, codes, scales, then
(only when they are random) the zero-points, then (int8 activations only) the row scales, then
(codebook weights only) the table of levels.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
from typing import Optional

import numpy as np
import torch

KIND_UINT, KIND_INT, KIND_FLOAT, KIND_CODEBOOK = 0, 1, 2, 3
_TORCH = {"f16": torch.float16, "bf16": torch.bfloat16}
E8M0_LO, E8M0_HI = 119, 130      # block-scale exponents drawn for "e8m0" scales: 2^-8 .. 2^3


@dataclass(frozen=True)
class Case:
    name: str
    M: int
    K: int
    N: int
    kind: int
    bits: int
    ebits: int = 0
    mbits: int = 0
    group: int = 128            # rows of W per scale; == K means per output channel
    act: str = "f16"            # dtype of A, C and of the de-quantised weights
    scale_dtype: str = "f16"
    zero: Optional[object] = None   # constant zero-point; "random": one draw per (group, column),
                                    # uniform over 0 .. zero_hi; None = no zero-point array
    zero_hi: Optional[int] = None   # largest random zero-point (default 2^bits - 1)
    a8: bool = False                # int8 activations: A is int8 with one fp32 scale per row; `act` is C's dtype
    scale_lo: float = 0.005
    scale_hi: float = 0.02
    seed: int = 0

    @property
    def wname(self) -> str:
        if self.kind == KIND_FLOAT:
            return f"f{self.bits}e{self.ebits}m{self.mbits}"
        if self.kind == KIND_CODEBOOK:
            return f"cb{self.bits}"
        return ("u" if self.kind == KIND_UINT else "i") + str(self.bits)


def _nonfinite_codes(case: Case):
    # the only non-finite encodings in the supported float families are the two
    # all-ones-magnitude codes of the 8-bit e4m3 format
    if case.kind == KIND_FLOAT and (case.ebits, case.mbits) == (4, 3):
        return (0x7F, 0xFF)
    return ()


def make_inputs(case: Case):
    """Returns dict(A, codes, scales, zeros).

    A      torch CPU tensor [M, K] of case.act, N(0,1) rounded to nearest even
    codes  numpy uint8 [K, N], the raw `bits`-bit patterns, uniform over the
           finite encodings (for intk: two's-complement patterns, i.e. values
           uniform over [-2^(k-1), 2^(k-1)-1])
    scales torch CPU tensor [K/group, N] of case.scale_dtype, U(lo, hi) -- for scale_dtype "e8m0"
           a uint8 tensor of exponents (the scale is 2^(e - 127))
    zeros  numpy uint8 [K/group, N] filled with case.zero -- or, for zero == "random",
           drawn uniformly from 0 .. zero_hi per (group, column) -- or None
    codebook  (kind KIND_CODEBOOK only) torch CPU fp16 [2^bits]: draws of N(0,1) clipped to +-3,
           sorted -- the unevenly spaced levels a learned companding quantiser ends up with for
           bell-shaped weights; codes are uniform indices into it
    """
    rng = np.random.Generator(np.random.PCG64(case.seed))
    A = torch.from_numpy(rng.standard_normal((case.M, case.K), dtype=np.float32))
    if case.a8:      # the same N(0,1) draw quantised to int8 at about 1/40 per step (saturating)
        A = torch.clamp(torch.round(A * 40.0), -127, 127).to(torch.int8)
    else:
        A = A.to(_TORCH[case.act])
    bad = _nonfinite_codes(case)
    if bad:
        ok = np.array([c for c in range(1 << case.bits) if c not in bad], dtype=np.uint8)
        codes = ok[rng.integers(0, ok.size, size=(case.K, case.N), dtype=np.uint8)]
    else:
        codes = rng.integers(0, 1 << case.bits, size=(case.K, case.N), dtype=np.uint8)
    G = case.K // case.group
    if case.scale_dtype == "e8m0":      # 8-bit exponents e (scale 2^(e - 127)), uniform over E8M0_LO .. E8M0_HI
        scales = torch.from_numpy(rng.integers(E8M0_LO, E8M0_HI + 1, size=(G, case.N), dtype=np.uint8))
    else:
        s = rng.uniform(case.scale_lo, case.scale_hi, size=(G, case.N)).astype(np.float32)
        scales = torch.from_numpy(s).to(_TORCH[case.scale_dtype])
    if case.zero is None:
        zeros = None
    elif case.zero == "random":
        hi = (1 << case.bits) - 1 if case.zero_hi is None else case.zero_hi
        zeros = rng.integers(0, hi + 1, size=(G, case.N), dtype=np.uint8)
    else:
        zeros = np.full((G, case.N), case.zero, dtype=np.uint8)
    out = {"A": A, "codes": codes, "scales": scales, "zeros": zeros}
    if case.a8:
        out["a_scale"] = torch.from_numpy(rng.uniform(0.02, 0.03, size=case.M).astype(np.float32))
    if case.kind == KIND_CODEBOOK:
        lv = np.sort(np.clip(rng.standard_normal(1 << case.bits), -3.0, 3.0)).astype(np.float32)
        out["codebook"] = torch.from_numpy(lv).to(torch.float16)
    return out


# ---- the five named configurations -----------------------------------------
def cfg1() -> Case:
    return Case("cfg1_u4_gemv", 1, 512, 512, KIND_UINT, 4, group=128, zero=8, seed=0)


def cfg2(M: int) -> Case:
    assert M in (1, 4, 16)
    return Case(f"cfg2_u3_decode_M{M}", M, 4096, 14336, KIND_UINT, 3, group=128, zero=4, seed=200 + M)


def cfg3(bits: int) -> Case:
    assert 1 <= bits <= 8
    return Case(f"cfg3_i{bits}_M16", 16, 8192, 28672, KIND_INT, bits, group=128, zero=None,
                scale_lo=0.002, scale_hi=0.02, seed=300 + bits)


_FLOATS = {4: (2, 1), 6: (3, 2), 8: (4, 3)}


def cfg4(bits: int, M: int) -> Case:
    e, m = _FLOATS[bits]
    return Case(f"cfg4_f{bits}e{e}m{m}_M{M}", M, 8192, 8192, KIND_FLOAT, bits, e, m, group=8192,
                act="bf16", scale_dtype="f16", zero=None, scale_lo=0.01, scale_hi=0.1,
                seed=400 + 10 * bits + ((1, 16, 64).index(M) if M in (1, 16, 64) else 3))   # other M: tables only


def cfg5(bits: int, M: int) -> Case:
    assert bits in (5, 6)
    return Case(f"cfg5_u{bits}_prefill_M{M}", M, 8192, 57344, KIND_UINT, bits, group=64,
                act="bf16", scale_dtype="bf16", zero=1 << (bits - 1),
                seed=500 + 10 * bits + ((1024, 4096).index(M) if M in (1024, 4096) else 2))   # other M: tables only


_SWEEP_FLOATS = {3: (1, 1), 4: (2, 1), 5: (2, 2), 6: (3, 2), 7: (3, 3), 8: (4, 3)}


def sweep(kind: int, bits: int, M: int = 16) -> Case:
    """The paper's full weight-type sweep (Figure "speedup over cuBLAS for every type"):
    M = 16, K = 8192, N = 57344, one scale per column group of 128; uint1..8 with a
    mid-range zero-point, int2..8, and the representative float of 3..8 bits."""
    if kind == KIND_FLOAT:
        e, m = _SWEEP_FLOATS[bits]
        return Case(f"sweep_f{bits}e{e}m{m}_M{M}", M, 8192, 57344, KIND_FLOAT, bits, e, m, group=128,
                    zero=None, scale_lo=0.01, scale_hi=0.1, seed=600 + bits)
    assert 1 <= bits <= 8
    if kind == KIND_UINT:
        return Case(f"sweep_u{bits}_M{M}", M, 8192, 57344, KIND_UINT, bits, group=128, zero=1 << (bits - 1),
                    seed=620 + bits)
    return Case(f"sweep_i{bits}_M{M}", M, 8192, 57344, KIND_INT, bits, group=128, zero=None,
                scale_lo=0.002, scale_hi=0.02, seed=640 + bits)


def codebook(bits: int, M: int = 16, act: str = "f16") -> Case:
    """Codebook-quantised weights on the type sweep's shape: K = 8192, N = 57344, group 128."""
    assert 1 <= bits <= 8
    return Case(f"codebook_{bits}_M{M}", M, 8192, 57344, KIND_CODEBOOK, bits, group=128, act=act,
                scale_dtype="f16", zero=None, seed=700 + bits)


def shrink(case: Case, **kw) -> Case:
    """Same recipe at another size (used by the element-by-element parity tests)."""
    return replace(case, **kw)

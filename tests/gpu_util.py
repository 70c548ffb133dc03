"""Helpers shared by the GPU parity tests: feed the same seeded bits to the HIP
library (through the C ABI binding) and to the CPU oracle."""
import numpy as np
import torch

from oracle import qgemm_oracle as O
from paper_2504_12984_amd import workloads as WL

ACT = {"f16": torch.float16, "bf16": torch.bfloat16}


def bits_of(t: torch.Tensor) -> np.ndarray:
    """uint16 bit patterns of an fp16/bf16 tensor (on any device)."""
    return t.detach().cpu().contiguous().view(torch.int16).numpy().view(np.uint16)


def to_f64(t: torch.Tensor) -> np.ndarray:
    return t.detach().cpu().to(torch.float64).numpy()


class Prepared:
    """One case on both sides: oracle-side arrays and device tensors."""

    def __init__(self, case: WL.Case, inputs=None):
        from paper_2504_12984_amd import binding as B
        self.case = case
        self.inp = inputs if inputs is not None else WL.make_inputs(case)
        c = case
        self.wtype = B.WType(c.kind, c.bits, c.ebits, c.mbits)
        self.stream = O.pack_canonical(self.inp["codes"], c.bits)             # oracle's canonical stream
        self.scales64 = to_f64(self.inp["scales"])
        self.A64 = to_f64(self.inp["A"])
        dev = "cuda:0"
        self.d_stream = torch.from_numpy(self.stream).to(dev)
        self.d_scales = self.inp["scales"].to(dev)
        self.d_zeros = None if self.inp["zeros"] is None else torch.from_numpy(self.inp["zeros"]).to(dev)
        self.d_A = self.inp["A"].to(dev)
        self.d_packed = B.repack(self.d_stream, self.wtype, c.K, c.N)
        self._packed = {0: self.d_packed}

    def packed(self, layout=0):
        from paper_2504_12984_amd import binding as B
        if layout not in self._packed:
            c = self.case
            self._packed[layout] = B.repack(self.d_stream, self.wtype, c.K, c.N, layout=layout)
        return self._packed[layout]

    def oracle_w(self):
        c = self.case
        return O.dequant_rounded(self.inp["codes"], c.kind, c.bits, c.ebits, c.mbits, self.scales64,
                                 self.inp["zeros"], c.group, c.act)

    def oracle_c(self, cols=None, rows=None):
        c = self.case
        A = self.A64 if rows is None else self.A64[rows]
        return O.qgemm_from_stream(A, self.stream, c.kind, c.bits, c.ebits, c.mbits, self.scales64,
                                   self.inp["zeros"], c.group, c.K, c.N, c.act, cols=cols)

    def gpu_w(self, layout=0):
        from paper_2504_12984_amd import binding as B
        c = self.case
        return B.qdequant(self.packed(layout), self.d_scales, self.d_zeros, self.wtype, ACT[c.act], c.group,
                          c.K, c.N, layout=layout)

    def gpu_c(self, A=None, layout=0):
        from paper_2504_12984_amd import binding as B
        c = self.case
        return B.qgemm(self.d_A if A is None else A, self.packed(layout), self.d_scales, self.d_zeros, self.wtype,
                       c.group, c.N, layout=layout)


def assert_c_close(C_gpu: torch.Tensor, C_ref: np.ndarray, what=""):
    """|C_gpu - C_ref| <= 1e-2 + 5e-3 |C_ref| elementwise (the stated tolerance)."""
    got = to_f64(C_gpu)
    ok = O.within_tolerance(got, C_ref)
    if not ok.all():
        bad = np.argwhere(~ok)
        i = tuple(bad[0])
        raise AssertionError(f"{what}: {len(bad)} of {ok.size} outside tolerance; first at {i}: "
                             f"gpu={got[i]!r} ref={C_ref[i]!r}")

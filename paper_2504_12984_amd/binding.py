"""ctypes binding of libqgemm.so -- argument marshalling only.

Every function has the name and argument order of its C entry point in
include/qgemm.h and takes torch CUDA tensors where the C call takes device
pointers.  Work is enqueued on torch's current stream.  There is no fallback:
if the library has not been built, importing this module raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
# QGEMM_LIB names another build of the same library (experiments with kernel variants)
LIB_PATH = os.environ.get("QGEMM_LIB") or os.path.join(_HERE, "libqgemm.so")

QG_OK, QG_EINVAL, QG_EUNSUPPORTED, QG_EHIP = 0, -1, -2, -3
QG_UINT, QG_INT, QG_FLOAT, QG_CODEBOOK = 0, 1, 2, 3
QG_F16, QG_BF16, QG_E8M0 = 0, 1, 2
QG_LAYOUT_TILE128x64 = 0
QG_LAYOUT_TILE128x64_R32 = 1
QG_LAYOUT_TILE128x64_I8 = 2
TILE_K, TILE_N = 128, 64

EXPORTS = ("qg_status_string", "qg_last_error", "qg_canonical_bytes", "qgemm_packed_bytes",
           "qg_pack_codes", "repack", "qdequant", "qgemm", "qgemm_noalloc", "qgemm_a8", "qdequant_codebook", "qgemm_codebook",
           "qg_set_knob", "qg_plan", "qg_probe_stream_read",
           "qg_probe_mfma")


class QgWType(ctypes.Structure):
    _fields_ = [("kind", ctypes.c_int32), ("bits", ctypes.c_int32),
                ("ebits", ctypes.c_int32), ("mbits", ctypes.c_int32)]


@dataclass(frozen=True)
class WType:
    kind: int
    bits: int
    ebits: int = 0
    mbits: int = 0

    def c(self) -> QgWType:
        return QgWType(self.kind, self.bits, self.ebits, self.mbits)


class QgError(RuntimeError):
    def __init__(self, fn: str, status: int):
        self.status = status
        msg = _lib.qg_status_string(status).decode()
        if status == QG_EHIP:
            msg += " (" + _lib.qg_last_error().decode() + ")"
        super().__init__(f"{fn}: {msg} [{status}]")


def _load() -> ctypes.CDLL:
    if not os.path.exists(LIB_PATH):
        raise ImportError(
            f"{LIB_PATH} is missing: build it with `python -m paper_2504_12984_amd.build` "
            "(there is no CPU fallback)")
    lib = ctypes.CDLL(LIB_PATH)
    vp, i32, i64, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64, ctypes.c_size_t
    lib.qg_status_string.restype = ctypes.c_char_p
    lib.qg_status_string.argtypes = [i32]
    lib.qg_last_error.restype = ctypes.c_char_p
    lib.qg_last_error.argtypes = []
    lib.qg_canonical_bytes.restype = sz
    lib.qg_canonical_bytes.argtypes = [i32, i64]
    lib.qgemm_packed_bytes.restype = sz
    lib.qgemm_packed_bytes.argtypes = [QgWType, i32, i64, i64]
    lib.qg_pack_codes.restype = i32
    lib.qg_pack_codes.argtypes = [vp, i32, i64, vp, vp]
    lib.repack.restype = i32
    lib.repack.argtypes = [vp, QgWType, i32, i64, i64, vp, vp]
    lib.qdequant.restype = i32
    lib.qdequant.argtypes = [vp, vp, vp, QgWType, i32, i32, i32, i64, i64, i64, vp, vp]
    lib.qgemm.restype = i32
    lib.qgemm.argtypes = [vp, vp, vp, vp, QgWType, i32, i32, i32, i64, i64, i64, i64, vp, vp]
    lib.qgemm_noalloc.restype = i32
    lib.qgemm_noalloc.argtypes = lib.qgemm.argtypes
    lib.qgemm_a8.restype = i32
    lib.qgemm_a8.argtypes = [vp, vp, vp, vp, vp, QgWType, i32, i32, i64, i64, i64, i64, vp, vp]
    lib.qdequant_codebook.restype = i32
    lib.qdequant_codebook.argtypes = [vp, vp, vp, i32, i32, i32, i64, i64, i64, vp, vp]
    lib.qgemm_codebook.restype = i32
    lib.qgemm_codebook.argtypes = [vp, vp, vp, vp, i32, i32, i32, i64, i64, i64, i64, vp, vp]
    lib.qg_set_knob.restype = i32
    lib.qg_plan.argtypes = [QgWType, i32, i32, i32, i64, i64, i64, i64, ctypes.POINTER(ctypes.c_int32)]
    lib.qg_plan.restype = i32
    lib.qg_set_knob.argtypes = [i32, i32]
    lib.qg_probe_stream_read.restype = i32
    lib.qg_probe_stream_read.argtypes = [vp, sz, vp, vp]
    lib.qg_probe_mfma.restype = i32
    lib.qg_probe_mfma.argtypes = [i32, i32, i32, i32, vp, ctypes.POINTER(ctypes.c_double), vp]
    return lib


_lib = _load()

_DT = {torch.float16: QG_F16, torch.bfloat16: QG_BF16}
# scale tensors may also be uint8: 8-bit exponents, one per 32 rows (microscaling block scales)
_SDT = {torch.float16: QG_F16, torch.bfloat16: QG_BF16, torch.uint8: QG_E8M0}


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _ptr(t, name):
    if t is None:
        return None
    if not (isinstance(t, torch.Tensor) and t.is_cuda and t.is_contiguous()):
        raise ValueError(f"{name} must be a contiguous CUDA tensor")
    return t.data_ptr()


def _check(fn, rc):
    if rc != QG_OK:
        raise QgError(fn, rc)


def qg_canonical_bytes(bits: int, count: int) -> int:
    return _lib.qg_canonical_bytes(bits, count)


def qgemm_packed_bytes(t: WType, K: int, N: int, layout: int = QG_LAYOUT_TILE128x64) -> int:
    return _lib.qgemm_packed_bytes(t.c(), layout, K, N)


def qg_pack_codes(codes: torch.Tensor, bits: int) -> torch.Tensor:
    """uint8 codes (any shape, row-major) -> canonical bit stream (uint8, 1-D)."""
    if codes.dtype != torch.uint8:
        raise ValueError("codes must be uint8")
    count = codes.numel()
    out = torch.empty(max(qg_canonical_bytes(bits, count), 1), dtype=torch.uint8, device=codes.device)
    _check("qg_pack_codes", _lib.qg_pack_codes(_ptr(codes, "codes"), bits, count, _ptr(out, "out"), _stream()))
    return out[:qg_canonical_bytes(bits, count)]


def repack(canonical: torch.Tensor, t: WType, K: int, N: int, layout: int = QG_LAYOUT_TILE128x64) -> torch.Tensor:
    """canonical [K,N] stream -> device layout (uint8, 1-D)."""
    nbytes = qgemm_packed_bytes(t, K, N, layout)
    if nbytes == 0:
        raise QgError("qgemm_packed_bytes", QG_EINVAL)
    if canonical.dtype != torch.uint8 or canonical.numel() < qg_canonical_bytes(t.bits, K * N):
        raise ValueError("canonical stream too short or not uint8")
    out = torch.empty(nbytes, dtype=torch.uint8, device=canonical.device)
    _check("repack", _lib.repack(_ptr(canonical, "canonical"), t.c(), layout, K, N, _ptr(out, "out"), _stream()))
    return out


def qdequant(packed: torch.Tensor, scales: torch.Tensor, zeros, t: WType, act: torch.dtype,
             group: int, K: int, N: int, layout: int = QG_LAYOUT_TILE128x64) -> torch.Tensor:
    out = torch.empty((K, N), dtype=act, device=packed.device)
    rc = _lib.qdequant(_ptr(packed, "packed"), _ptr(scales, "scales"), _ptr(zeros, "zeros"), t.c(), layout,
                       _DT[act], _SDT[scales.dtype], group, K, N, _ptr(out, "out"), _stream())
    _check("qdequant", rc)
    return out


def qgemm(A: torch.Tensor, packed: torch.Tensor, scales: torch.Tensor, zeros, t: WType, group: int,
          N: int, out: torch.Tensor | None = None, layout: int = QG_LAYOUT_TILE128x64,
          entry: str = "qgemm") -> torch.Tensor:
    """C[M,N] = A[M,K] . dequant(W); dtype of A is the activation dtype.  `entry` names the C
    entry point ("qgemm" or "qgemm_noalloc"; with the latter pass `out`, or this wrapper's
    torch.empty allocates)."""
    if A.dim() != 2 or A.dtype not in _DT:
        raise ValueError("A must be [M,K] fp16 or bf16")
    M, K = A.shape
    rows = K // group if group > 0 else 1                    # group 0 = one scale per output column
    if scales.dtype not in _SDT or tuple(scales.shape) != (rows, N):
        raise ValueError("scales must be [K/group, N] fp16 or bf16 (or uint8 exponents for block scales)")
    if zeros is not None and (zeros.dtype != torch.uint8 or tuple(zeros.shape) != (rows, N)):
        raise ValueError("zeros must be uint8 [K/group, N]")
    if out is None:
        out = torch.empty((M, N), dtype=A.dtype, device=A.device)
    fn = {"qgemm": _lib.qgemm, "qgemm_noalloc": _lib.qgemm_noalloc}[entry]
    rc = fn(_ptr(A, "A"), _ptr(packed, "packed"), _ptr(scales, "scales"), _ptr(zeros, "zeros"), t.c(),
            layout, _DT[A.dtype], _SDT[scales.dtype], group, M, N, K, _ptr(out, "C"), _stream())
    _check(entry, rc)
    return out


def qgemm_noalloc(A: torch.Tensor, packed: torch.Tensor, scales: torch.Tensor, zeros, t: WType, group: int,
                  N: int, out: torch.Tensor, layout: int = QG_LAYOUT_TILE128x64) -> torch.Tensor:
    """qgemm through the entry point that allocates nothing (the output is the caller's)."""
    return qgemm(A, packed, scales, zeros, t, group, N, out=out, layout=layout, entry="qgemm_noalloc")


def qgemm_a8(A8: torch.Tensor, a_scale, packed: torch.Tensor, scales: torch.Tensor, zeros, t: WType, group: int,
             N: int, out_dtype: torch.dtype = torch.float16, out: torch.Tensor | None = None) -> torch.Tensor:
    """C[M,N] = a_scale[m] * sum_g s[g,n] * (A8 . (codes - z))_g; A8 int8 [M,K], a_scale fp32 [M] or None,
    `packed` in QG_LAYOUT_TILE128x64_I8."""
    if A8.dim() != 2 or A8.dtype != torch.int8:
        raise ValueError("A8 must be [M,K] int8")
    M, K = A8.shape
    rows = K // group if group > 0 else 1
    if scales.dtype not in _DT or tuple(scales.shape) != (rows, N):
        raise ValueError("scales must be [K/group, N] fp16 or bf16 (or uint8 exponents for block scales)")
    if zeros is not None and (zeros.dtype != torch.uint8 or tuple(zeros.shape) != (rows, N)):
        raise ValueError("zeros must be uint8 [K/group, N]")
    if a_scale is not None and (a_scale.dtype != torch.float32 or tuple(a_scale.shape) != (M,)):
        raise ValueError("a_scale must be fp32 [M]")
    if out is None:
        out = torch.empty((M, N), dtype=out_dtype, device=A8.device)
    rc = _lib.qgemm_a8(_ptr(A8, "A8"), _ptr(a_scale, "a_scale"), _ptr(packed, "packed"), _ptr(scales, "scales"),
                       _ptr(zeros, "zeros"), t.c(), _DT[out.dtype], _DT[scales.dtype], group, M, N, K, _ptr(out, "C"),
                       _stream())
    _check("qgemm_a8", rc)
    return out


class BoundQgemm:
    """One qgemm call with its arguments checked and marshalled once.

    For callers that issue the same matmul many times (a decode loop, the
    benchmark): `__call__` is a single foreign call on pre-built C arguments, a
    few microseconds cheaper than `qgemm`, which matters when the kernel itself
    takes under ten.  The tensors are held by reference and must stay alive and
    in place; the stream is the one current when the object was made unless one
    is passed.
    """

    def __init__(self, A: torch.Tensor, packed: torch.Tensor, scales: torch.Tensor, zeros, t: WType, group: int,
                 N: int, out: torch.Tensor, layout: int = QG_LAYOUT_TILE128x64, stream: int | None = None,
                 entry: str = "qgemm"):
        self._fn = {"qgemm": _lib.qgemm, "qgemm_noalloc": _lib.qgemm_noalloc}[entry]
        self._entry = entry
        if A.dim() != 2 or A.dtype not in _DT:
            raise ValueError("A must be [M,K] fp16 or bf16")
        M, K = A.shape
        rows = K // group if group > 0 else 1                    # group 0 = one scale per output column
        if scales.dtype not in _SDT or tuple(scales.shape) != (rows, N):
            raise ValueError("scales must be [K/group, N] fp16 or bf16 (or uint8 exponents for block scales)")
        if zeros is not None and (zeros.dtype != torch.uint8 or tuple(zeros.shape) != (rows, N)):
            raise ValueError("zeros must be uint8 [K/group, N]")
        if tuple(out.shape) != (M, N) or out.dtype != A.dtype:
            raise ValueError("out must be [M,N] of A's dtype")
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        self._keep = (A, packed, scales, zeros, out)
        self.out = out
        self._args = (vp(_ptr(A, "A")), vp(_ptr(packed, "packed")), vp(_ptr(scales, "scales")),
                      vp(_ptr(zeros, "zeros")), t.c(), i32(layout), i32(_DT[A.dtype]), i32(_SDT[scales.dtype]),
                      i64(group), i64(M), i64(N), i64(K), vp(_ptr(out, "C")),
                      vp(_stream() if stream is None else stream))

    def __call__(self) -> torch.Tensor:
        rc = self._fn(*self._args)
        if rc != QG_OK:
            raise QgError(self._entry, rc)
        return self.out


class BoundQgemmA8:
    """One qgemm_a8 call with its arguments checked and marshalled once (see BoundQgemm)."""

    def __init__(self, A8: torch.Tensor, a_scale, packed: torch.Tensor, scales: torch.Tensor, zeros, t: WType,
                 group: int, N: int, out: torch.Tensor, stream: int | None = None):
        if A8.dim() != 2 or A8.dtype != torch.int8:
            raise ValueError("A8 must be [M,K] int8")
        M, K = A8.shape
        rows = K // group if group > 0 else 1
        if scales.dtype not in _DT or tuple(scales.shape) != (rows, N):
            raise ValueError("scales must be [K/group, N] fp16 or bf16 (or uint8 exponents for block scales)")
        if zeros is not None and (zeros.dtype != torch.uint8 or tuple(zeros.shape) != (rows, N)):
            raise ValueError("zeros must be uint8 [K/group, N]")
        if a_scale is not None and (a_scale.dtype != torch.float32 or tuple(a_scale.shape) != (M,)):
            raise ValueError("a_scale must be fp32 [M]")
        if tuple(out.shape) != (M, N) or out.dtype not in _DT:
            raise ValueError("out must be [M,N] fp16 or bf16")
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        self._keep = (A8, a_scale, packed, scales, zeros, out)
        self.out = out
        self._args = (vp(_ptr(A8, "A8")), vp(_ptr(a_scale, "a_scale")), vp(_ptr(packed, "packed")),
                      vp(_ptr(scales, "scales")), vp(_ptr(zeros, "zeros")), t.c(), i32(_DT[out.dtype]),
                      i32(_DT[scales.dtype]), i64(group), i64(M), i64(N), i64(K), vp(_ptr(out, "C")),
                      vp(_stream() if stream is None else stream))

    def __call__(self) -> torch.Tensor:
        rc = _lib.qgemm_a8(*self._args)
        if rc != QG_OK:
            raise QgError("qgemm_a8", rc)
        return self.out


def _check_codebook(codebook: torch.Tensor, bits: int):
    if not (1 <= bits <= 8):
        raise ValueError("bits must be 1..8")
    if codebook.dtype != torch.float16 or tuple(codebook.shape) != (1 << bits,):
        raise ValueError("codebook must be fp16 [2^bits]")


def qdequant_codebook(packed: torch.Tensor, codebook: torch.Tensor, scales: torch.Tensor, bits: int, act: torch.dtype,
                      group: int, K: int, N: int) -> torch.Tensor:
    """W_out[K,N] = rne_act(codebook[code] * scale); `packed` = repack of WType(QG_CODEBOOK, bits)."""
    _check_codebook(codebook, bits)
    out = torch.empty((K, N), dtype=act, device=packed.device)
    rc = _lib.qdequant_codebook(_ptr(packed, "packed"), _ptr(codebook, "codebook"), _ptr(scales, "scales"), bits,
                                _DT[act], _DT[scales.dtype], group, K, N, _ptr(out, "out"), _stream())
    _check("qdequant_codebook", rc)
    return out


def qgemm_codebook(A: torch.Tensor, packed: torch.Tensor, codebook: torch.Tensor, scales: torch.Tensor, bits: int,
                   group: int, N: int, out: torch.Tensor | None = None) -> torch.Tensor:
    """C[M,N] = A[M,K] . rne_act(codebook[code] * scale); dtype of A is the activation dtype."""
    if A.dim() != 2 or A.dtype not in _DT:
        raise ValueError("A must be [M,K] fp16 or bf16")
    _check_codebook(codebook, bits)
    M, K = A.shape
    rows = K // group if group > 0 else 1
    if scales.dtype not in _DT or tuple(scales.shape) != (rows, N):
        raise ValueError("scales must be [K/group, N] fp16 or bf16")
    if out is None:
        out = torch.empty((M, N), dtype=A.dtype, device=A.device)
    rc = _lib.qgemm_codebook(_ptr(A, "A"), _ptr(packed, "packed"), _ptr(codebook, "codebook"), _ptr(scales, "scales"), bits,
                             _DT[A.dtype], _DT[scales.dtype], group, M, N, K, _ptr(out, "C"), _stream())
    _check("qgemm_codebook", rc)
    return out


class BoundQgemmCodebook:
    """One qgemm_codebook call with its arguments checked and marshalled once (see BoundQgemm)."""

    def __init__(self, A: torch.Tensor, packed: torch.Tensor, codebook: torch.Tensor, scales: torch.Tensor, bits: int,
                 group: int, N: int, out: torch.Tensor, stream: int | None = None):
        if A.dim() != 2 or A.dtype not in _DT:
            raise ValueError("A must be [M,K] fp16 or bf16")
        _check_codebook(codebook, bits)
        M, K = A.shape
        rows = K // group if group > 0 else 1
        if scales.dtype not in _DT or tuple(scales.shape) != (rows, N):
            raise ValueError("scales must be [K/group, N] fp16 or bf16")
        if tuple(out.shape) != (M, N) or out.dtype != A.dtype:
            raise ValueError("out must be [M,N] of A's dtype")
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
        self._keep = (A, packed, codebook, scales, out)
        self.out = out
        self._args = (vp(_ptr(A, "A")), vp(_ptr(packed, "packed")), vp(_ptr(codebook, "codebook")),
                      vp(_ptr(scales, "scales")), i32(bits), i32(_DT[A.dtype]), i32(_DT[scales.dtype]),
                      i64(group), i64(M), i64(N), i64(K), vp(_ptr(out, "C")),
                      vp(_stream() if stream is None else stream))

    def __call__(self) -> torch.Tensor:
        rc = _lib.qgemm_codebook(*self._args)
        if rc != QG_OK:
            raise QgError("qgemm_codebook", rc)
        return self.out


def qg_probe_stream_read(buf: torch.Tensor, sink: torch.Tensor):
    """The read-only streaming probe over all of `buf` (measurement aid).  Returns a
    callable that enqueues it on the stream current now; like BoundQgemm, the
    arguments are marshalled once so that the call costs the host as little as a
    bound matmul call."""
    vp = ctypes.c_void_p
    args = (vp(_ptr(buf, "buf")), ctypes.c_size_t(buf.numel() * buf.element_size()), vp(_ptr(sink, "sink")),
            vp(_stream()))

    def call():
        _check("qg_probe_stream_read", _lib.qg_probe_stream_read(*args))
    call.keep = (buf, sink)
    return call


def qg_probe_mfma(bf16: bool, random_data: bool, iters: int, waves_per_simd: int, sink: torch.Tensor) -> float:
    """Enqueue the register-resident matrix-instruction probe; returns its flop count."""
    flops = ctypes.c_double(0.0)
    _check("qg_probe_mfma", _lib.qg_probe_mfma(int(bf16), int(random_data), iters, waves_per_simd,
                                               _ptr(sink, "sink"), ctypes.byref(flops), _stream()))
    return flops.value


def qg_set_knob(knob: int, value: int) -> int:
    return _lib.qg_set_knob(knob, value)


def qg_plan(t: WType, group: int, M: int, N: int, K: int, act: int = QG_F16, scale_dtype: int | None = None,
            layout: int = QG_LAYOUT_TILE128x64) -> dict:
    """What qgemm would launch for this shape (host arithmetic only, no GPU needed)."""
    out = (ctypes.c_int32 * 5)()
    _check("qg_plan", _lib.qg_plan(t.c(), layout, act, act if scale_dtype is None else scale_dtype, group, M, N, K, out))
    return {"path": out[0], "variant": out[1], "row_tile": out[2], "splitk": out[3], "chunks_per_slab": out[4]}

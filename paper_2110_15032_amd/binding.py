"""ctypes binding with the same names as the C ABI (include/sbp.h)."""
from __future__ import annotations

import ctypes
import os
from typing import Sequence

HERE = os.path.dirname(os.path.abspath(__file__))
# SBP_LIB names an alternative build of the same library (development / timing experiments)
_LIB_PATH = os.environ.get("SBP_LIB") or os.path.join(HERE, "libsbp_mi355x.so")

# signatures (sbp_t)
def S(axis: int) -> int:
    return int(axis)
B = -1
P_SUM = -2
P_MAX = -3
AUTO = -100
# dtypes
F32 = 0
BF16 = 1
I32 = 2
# epilogues
EPI_NONE = 0
EPI_GELU = 1
# knobs
KNOB_GEMM_VARIANT = 0
KNOB_TILE_ORDER = 1
KNOB_BOX_REDUCE = 2

#: every symbol include/sbp.h declares
EXPORTS = ("sbp_infer_matmul", "sbp_local_shape", "sbp_matmul", "sbp_matmul_ex", "sbp_matmul_rowmax", "sbp_boxing", "sbp_boxing_across", "sbp_boxing_cast",
           "sbp_infer_matmul_2d", "sbp_local_shape_2d", "sbp_matmul_2d", "sbp_boxing_2d",
           "sbp_row_max", "sbp_row_sumexp", "sbp_xent_loss", "sbp_xent_grad", "sbp_set_knob", "sbp_probe_mfma", "sbp_probe_mfma_static", "sbp_strerror")


class _CTensor(ctypes.Structure):
    _fields_ = [("shard", ctypes.POINTER(ctypes.c_void_p)),
                ("rows", ctypes.c_int64), ("cols", ctypes.c_int64),
                ("dtype", ctypes.c_int32), ("trans", ctypes.c_int32), ("ld", ctypes.c_int64)]


class SbpError(RuntimeError):
    def __init__(self, status: int, what: str):
        super().__init__(f"{what}: status {status} ({sbp_strerror(status)})")
        self.status = status


_lib = None


def lib_path() -> str:
    return _LIB_PATH


def lib() -> ctypes.CDLL:
    """Load libsbp_mi355x.so.  There is no fallback: without the library nothing runs."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise ImportError(f"{_LIB_PATH} is missing: build it with `python -m paper_2110_15032_amd.build`")
        # PyTorch ships its own copy of the HIP runtime.  Callers hand this library device memory and
        # streams that PyTorch owns, so both must sit on ONE runtime: let PyTorch's load first (the
        # library's dependency then resolves to it); loaded the other way round, this library's
        # launches go to a second runtime that does not know the device PyTorch has opened.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        L = ctypes.CDLL(_LIB_PATH)
        i32, i64, vp = ctypes.c_int32, ctypes.c_int64, ctypes.c_void_p
        T = ctypes.POINTER(_CTensor)
        L.sbp_infer_matmul.argtypes = [i32, i32, ctypes.POINTER(i32)]
        L.sbp_local_shape.argtypes = [i64, i64, i32, i32, i32, ctypes.POINTER(i64), ctypes.POINTER(i64)]
        L.sbp_matmul.argtypes = [T, i32, T, i32, T, i32, i32, vp]
        L.sbp_matmul_ex.argtypes = [T, i32, T, i32, T, i32, i32, vp, i32]
        L.sbp_matmul_rowmax.argtypes = [T, i32, T, i32, T, i32, T, i32, vp]
        L.sbp_boxing.argtypes = [T, i32, T, i32, i32, vp]
        L.sbp_boxing_across.argtypes = [T, i32, i32, T, i32, i32, vp]
        L.sbp_boxing_cast.argtypes = [T, i32, T, i32, i32, vp]
        P2 = ctypes.POINTER(i32)
        L.sbp_infer_matmul_2d.argtypes = [P2, P2, P2]
        L.sbp_local_shape_2d.argtypes = [i64, i64, P2, i32, i32, i32, i32, ctypes.POINTER(i64), ctypes.POINTER(i64)]
        L.sbp_matmul_2d.argtypes = [T, P2, T, P2, T, P2, i32, i32, vp]
        L.sbp_boxing_2d.argtypes = [T, P2, T, P2, i32, i32, vp]
        L.sbp_row_max.argtypes = [T, i32, T, i32, vp]
        L.sbp_row_sumexp.argtypes = [T, i32, T, T, i32, vp]
        L.sbp_xent_loss.argtypes = [T, i32, T, T, T, T, i32, vp]
        L.sbp_xent_grad.argtypes = [T, i32, T, T, T, T, T, i32, vp]
        L.sbp_set_knob.argtypes = [i32, i32]
        L.sbp_probe_mfma.argtypes = [i32, i32, i32, vp, vp]
        L.sbp_probe_mfma_static.argtypes = [i32, i32, i32, vp, vp]
        L.sbp_strerror.argtypes = [i32]
        L.sbp_strerror.restype = ctypes.c_char_p
        for f in EXPORTS[:-1]:
            getattr(L, f).restype = i32
        _lib = L
    return _lib


class SbpTensor:
    """A global tensor as the ABI sees it: k device pointers + global shape + dtype + trans + row pitch
    (`ld` elements between stored rows, 0 = dense).

    `shards` are integers (device addresses) or objects with .data_ptr() (torch tensors); the
    object keeps them alive.  Nothing is copied."""

    def __init__(self, shards: Sequence, rows: int, cols: int, dtype: int, trans: int = 0, ld: int = 0):
        self.keep = list(shards)
        ptrs = [s if isinstance(s, int) or s is None else s.data_ptr() for s in shards]
        self.k = len(ptrs)
        self._arr = (ctypes.c_void_p * max(1, self.k))(*ptrs)
        self.c = _CTensor(ctypes.cast(self._arr, ctypes.POINTER(ctypes.c_void_p)), rows, cols, dtype, trans, ld)

    def ref(self):
        return ctypes.byref(self.c)


def _stream_ptr(stream) -> ctypes.c_void_p:
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    return ctypes.c_void_p(stream)


def _need(k: int, *tensors) -> None:
    """The library reads k pointers from every shard array it is given: refuse here, before the call,
    a tensor that holds fewer (a count the library itself rejects is left to the library)."""
    if not 1 <= k <= 64:
        return
    for t in tensors:
        if t is not None and t.k < k:
            raise ValueError(f"tensor holds {t.k} shard pointers, the call needs {k}")


def _check(status: int, what: str) -> None:
    if status != 0:
        raise SbpError(status, what)


def sbp_strerror(status: int) -> str:
    return lib().sbp_strerror(status).decode()


def sbp_infer_matmul(sbp_x: int, sbp_w: int) -> int:
    out = ctypes.c_int32()
    _check(lib().sbp_infer_matmul(sbp_x, sbp_w, ctypes.byref(out)), "sbp_infer_matmul")
    return out.value


def sbp_local_shape(rows: int, cols: int, sbp: int, k: int, i: int) -> tuple[int, int]:
    r, c = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().sbp_local_shape(rows, cols, sbp, k, i, ctypes.byref(r), ctypes.byref(c)), "sbp_local_shape")
    return r.value, c.value


def sbp_matmul(x: SbpTensor, sbp_x: int, w: SbpTensor, sbp_w: int, y: SbpTensor, sbp_y: int, k: int,
               stream=None) -> None:
    _need(k, x, w, y)
    _check(lib().sbp_matmul(x.ref(), sbp_x, w.ref(), sbp_w, y.ref(), sbp_y, k, _stream_ptr(stream)), "sbp_matmul")


def sbp_matmul_ex(x: SbpTensor, sbp_x: int, w: SbpTensor, sbp_w: int, y: SbpTensor, sbp_y: int, k: int,
                  stream=None, epilogue: int = EPI_NONE) -> None:
    _need(k, x, w, y)
    _check(lib().sbp_matmul_ex(x.ref(), sbp_x, w.ref(), sbp_w, y.ref(), sbp_y, k, _stream_ptr(stream), epilogue),
           "sbp_matmul_ex")


def sbp_matmul_rowmax(x: SbpTensor, sbp_x: int, w: SbpTensor, sbp_w: int, y: SbpTensor, sbp_y: int, rowmax: SbpTensor,
                      k: int, stream=None) -> None:
    _need(k, x, w, y, rowmax)
    _check(lib().sbp_matmul_rowmax(x.ref(), sbp_x, w.ref(), sbp_w, y.ref(), sbp_y, rowmax.ref(), k, _stream_ptr(stream)),
           "sbp_matmul_rowmax")


def sbp_boxing(inp: SbpTensor, sbp_in: int, out: SbpTensor, sbp_out: int, k: int, stream=None) -> None:
    _need(k, inp, out)
    _check(lib().sbp_boxing(inp.ref(), sbp_in, out.ref(), sbp_out, k, _stream_ptr(stream)), "sbp_boxing")


def sbp_boxing_across(inp: SbpTensor, sbp_in: int, k_in: int, out: SbpTensor, sbp_out: int, k_out: int, stream=None) -> None:
    _need(k_in, inp)
    _need(k_out, out)
    _check(lib().sbp_boxing_across(inp.ref(), sbp_in, k_in, out.ref(), sbp_out, k_out, _stream_ptr(stream)),
           "sbp_boxing_across")


def sbp_boxing_cast(inp: SbpTensor, sbp_in: int, out: SbpTensor, sbp_out: int, k: int, stream=None) -> None:
    _need(k, inp, out)
    _check(lib().sbp_boxing_cast(inp.ref(), sbp_in, out.ref(), sbp_out, k, _stream_ptr(stream)), "sbp_boxing_cast")


def _pair(s):
    return (ctypes.c_int32 * 2)(int(s[0]), int(s[1]))


def sbp_infer_matmul_2d(sbp_x, sbp_w):
    y = (ctypes.c_int32 * 2)()
    _check(lib().sbp_infer_matmul_2d(_pair(sbp_x), _pair(sbp_w), y), "sbp_infer_matmul_2d")
    return (y[0], y[1])


def sbp_local_shape_2d(rows: int, cols: int, sbp2, k0: int, k1: int, a: int, b: int):
    lr, lc = ctypes.c_int64(), ctypes.c_int64()
    _check(lib().sbp_local_shape_2d(rows, cols, _pair(sbp2), k0, k1, a, b, ctypes.byref(lr), ctypes.byref(lc)),
           "sbp_local_shape_2d")
    return lr.value, lc.value


def sbp_matmul_2d(x: SbpTensor, sbp_x, w: SbpTensor, sbp_w, y: SbpTensor, sbp_y, k0: int, k1: int, stream=None) -> None:
    _need(k0 * k1, x, w, y)
    sy = _pair(sbp_y) if sbp_y is not None else None
    _check(lib().sbp_matmul_2d(x.ref(), _pair(sbp_x), w.ref(), _pair(sbp_w), y.ref(), sy, k0, k1, _stream_ptr(stream)),
           "sbp_matmul_2d")


def sbp_boxing_2d(inp: SbpTensor, sbp_in, out: SbpTensor, sbp_out, k0: int, k1: int, stream=None) -> None:
    _need(k0 * k1, inp, out)
    _check(lib().sbp_boxing_2d(inp.ref(), _pair(sbp_in), out.ref(), _pair(sbp_out), k0, k1, _stream_ptr(stream)),
           "sbp_boxing_2d")


def sbp_row_max(logits: SbpTensor, sbp_l: int, out: SbpTensor, k: int, stream=None) -> None:
    _need(k, logits, out)
    _check(lib().sbp_row_max(logits.ref(), sbp_l, out.ref(), k, _stream_ptr(stream)), "sbp_row_max")


def sbp_row_sumexp(logits: SbpTensor, sbp_l: int, gmax: SbpTensor, out: SbpTensor, k: int, stream=None) -> None:
    _need(k, logits, gmax, out)
    _check(lib().sbp_row_sumexp(logits.ref(), sbp_l, gmax.ref(), out.ref(), k, _stream_ptr(stream)), "sbp_row_sumexp")


def sbp_xent_loss(logits: SbpTensor, sbp_l: int, labels: SbpTensor, gmax: SbpTensor, denom: SbpTensor, loss: SbpTensor,
                  k: int, stream=None) -> None:
    _need(k, logits, labels, gmax, denom, loss)
    _check(lib().sbp_xent_loss(logits.ref(), sbp_l, labels.ref(), gmax.ref(), denom.ref(), loss.ref(), k,
                               _stream_ptr(stream)), "sbp_xent_loss")


def sbp_xent_grad(logits: SbpTensor, sbp_l: int, labels: SbpTensor, gmax: SbpTensor, denom: SbpTensor, grad: SbpTensor,
                  dlogits: SbpTensor, k: int, stream=None) -> None:
    _need(k, logits, labels, gmax, denom, grad, dlogits)
    _check(lib().sbp_xent_grad(logits.ref(), sbp_l, labels.ref(), gmax.ref(), denom.ref(), grad.ref(), dlogits.ref(), k,
                               _stream_ptr(stream)), "sbp_xent_grad")


def sbp_probe_mfma(mode: int, iters: int, zero_operands: int, scratch, stream=None) -> None:
    ptr = scratch if isinstance(scratch, int) else scratch.data_ptr()
    _check(lib().sbp_probe_mfma(mode, iters, zero_operands, ctypes.c_void_p(ptr), _stream_ptr(stream)), "sbp_probe_mfma")


def sbp_probe_mfma_static(mode: int, iters: int, zero_operands: int, out, stream=None) -> None:
    ptr = out if isinstance(out, int) else out.data_ptr()
    _check(lib().sbp_probe_mfma_static(mode, iters, zero_operands, ctypes.c_void_p(ptr), _stream_ptr(stream)), "sbp_probe_mfma_static")


def sbp_set_knob(knob: int, value: int) -> None:
    _check(lib().sbp_set_knob(knob, value), "sbp_set_knob")

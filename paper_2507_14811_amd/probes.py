"""ctypes binding of libsegquant_probes.so (include/segquant_probes.h): benchmark probes, same names as the C ABI.

Argument marshalling only.  The probes are not part of the quantized layer; only the benchmark loads them."""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libsegquant_probes.so")
EXPORTS = ("sqp_mfma", "sqp_mfma_fp8", "sqp_launch", "sqp_roundtrip", "sqp_copy")
_lib = None


def load_library() -> C.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2507_14811_amd.build`")
    import torch  # noqa: F401  loads the HIP runtime the library binds to

    lib = C.CDLL(LIB_PATH)
    vp, i32 = C.c_void_p, C.c_int
    lib.sqp_mfma.argtypes = [vp, C.c_size_t, i32, C.POINTER(C.c_double), vp]
    lib.sqp_mfma_fp8.argtypes = [vp, C.c_size_t, i32, C.POINTER(C.c_double), vp]
    lib.sqp_launch.argtypes = [i32, i32, i32, vp]
    lib.sqp_roundtrip.argtypes = [vp, vp, i32, i32, vp]
    lib.sqp_copy.argtypes = [vp, vp, C.c_size_t, vp]
    for name in EXPORTS:
        getattr(lib, name).restype = i32
    _lib = lib
    return lib


def _stream(stream):
    import torch

    return C.c_void_p((stream if stream is not None else torch.cuda.current_stream()).cuda_stream)


def _check(rc: int, what: str) -> None:
    if rc != 0:
        raise RuntimeError(f"{what} failed with status {rc}")


def sqp_mfma(codes, iters: int, stream=None) -> float:
    """Launches the register-only int8 MFMA loop on int8 device tensor `codes`; returns the ops of one launch."""
    ops = C.c_double(0.0)
    _check(load_library().sqp_mfma(codes.data_ptr(), codes.numel(), int(iters), C.byref(ops), _stream(stream)), "sqp_mfma")
    return float(ops.value)


def sqp_mfma_fp8(codes, iters: int, stream=None) -> float:
    """The same loop on the fp8 matrix cores, `codes` read as E4M3 bytes; returns the flops of one launch."""
    ops = C.c_double(0.0)
    _check(load_library().sqp_mfma_fp8(codes.data_ptr(), codes.numel(), int(iters), C.byref(ops), _stream(stream)), "sqp_mfma_fp8")
    return float(ops.value)


def sqp_launch(grid: int, block: int, lds_bytes: int = 0, stream=None) -> None:
    _check(load_library().sqp_launch(int(grid), int(block), int(lds_bytes), _stream(stream)), "sqp_launch")


def sqp_roundtrip(src, dst, grid: int, block: int, stream=None) -> None:
    assert src.numel() >= grid * block and dst.numel() >= grid * block and src.element_size() == 4
    _check(load_library().sqp_roundtrip(src.data_ptr(), dst.data_ptr(), int(grid), int(block), _stream(stream)), "sqp_roundtrip")


def sqp_copy(src, dst, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() >= nbytes
    _check(load_library().sqp_copy(src.data_ptr(), dst.data_ptr(), nbytes, _stream(stream)), "sqp_copy")

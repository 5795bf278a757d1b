"""ctypes binding over libsrft_measure.so: the measurement aids declared in ``include/srft_measure.h``
(plain streaming kernels; not part of the method).  Used by bench.py only."""
from __future__ import annotations

import ctypes as C
import os

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libsrft_measure.so")
EXPORTS = ["srft_stream_copy", "srft_stream_mix", "srft_measure_last_hip_error"]
_lib = None


def lib() -> C.CDLL:
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with `python -m paper_2605_05699_amd.build`")
        L = C.CDLL(LIB_PATH)
        vp, i64, ci = C.c_void_p, C.c_int64, C.c_int
        L.srft_stream_copy.argtypes = [vp, vp, i64, vp]
        L.srft_stream_mix.argtypes = [vp, vp, i64, ci, ci, ci, ci, vp]
        L.srft_measure_last_hip_error.argtypes = []
        for name in EXPORTS:
            getattr(L, name).restype = ci
        _lib = L
    return _lib


def _check(status: int, where: str) -> None:
    if status != 0:
        raise RuntimeError(f"{where}: status {status} [hipError {lib().srft_measure_last_hip_error()}]")


def _stream_handle(stream) -> int:
    return int((stream or torch.cuda.current_stream()).cuda_stream)


def srft_stream_copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    nbytes = src.numel() * src.element_size()
    assert dst.numel() * dst.element_size() == nbytes and dst.is_cuda and src.is_cuda
    _check(lib().srft_stream_copy(dst.data_ptr(), src.data_ptr(), nbytes, _stream_handle(stream)), "srft_stream_copy")


def srft_stream_mix(src: torch.Tensor, dst: torch.Tensor, n_tiles: int, read_bytes: int, write_bytes: int,
                    workgroups: int = 0, nontemporal=False, stream=None) -> None:
    """nontemporal: bool, or the access bit set of the C entry point (1 non-temporal, 2 = 64 bytes per lane, 4 = a contiguous eighth of the tiles per die)."""
    assert src.is_cuda and dst.is_cuda
    assert src.numel() * src.element_size() >= n_tiles * read_bytes
    assert dst.numel() * dst.element_size() >= n_tiles * write_bytes
    _check(lib().srft_stream_mix(src.data_ptr(), dst.data_ptr(), n_tiles, read_bytes, write_bytes, workgroups,
                                 int(nontemporal), _stream_handle(stream)), "srft_stream_mix")

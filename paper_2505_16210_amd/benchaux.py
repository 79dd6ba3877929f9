"""ctypes binding of libnqkv_benchaux (include/nqkv_benchaux.h): measurement helpers for bench.py
-- a plain read stream, a plain copy of known size, a plain read : write mix, an empty kernel.  Not part of the method and
not loaded by the product binding."""
from __future__ import annotations

import ctypes
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnqkv_benchaux.so")
PROBE_WORKGROUPS = 4096
EXPORTS = ("nqkv_aux_read_stream", "nqkv_aux_copy", "nqkv_aux_empty_launch", "nqkv_aux_mix_stream")

if not os.path.exists(LIB_PATH):
    raise ImportError("libnqkv_benchaux.so is not built: run python paper_2505_16210_amd/build.py")
lib = ctypes.CDLL(LIB_PATH)
lib.nqkv_aux_read_stream.restype = ctypes.c_int
lib.nqkv_aux_read_stream.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_void_p]
lib.nqkv_aux_copy.restype = ctypes.c_int
lib.nqkv_aux_copy.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p]
lib.nqkv_aux_mix_stream.restype = ctypes.c_int
lib.nqkv_aux_mix_stream.argtypes = [ctypes.c_void_p, ctypes.c_size_t, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int,
                                    ctypes.c_int, ctypes.POINTER(ctypes.c_size_t), ctypes.c_void_p]
lib.nqkv_aux_empty_launch.restype = ctypes.c_int
lib.nqkv_aux_empty_launch.argtypes = [ctypes.c_void_p]


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def read_stream(src: torch.Tensor, checksums: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """One read pass over `src` (contiguous, bytes % 16 == 0) -> int32 [PROBE_WORKGROUPS] xor checksums."""
    assert src.is_contiguous()
    if checksums is None:
        checksums = torch.empty(PROBE_WORKGROUPS, dtype=torch.int32, device=src.device)
    rc = lib.nqkv_aux_read_stream(src.data_ptr(), src.numel() * src.element_size(), checksums.data_ptr(), _stream(stream))
    if rc:
        raise RuntimeError("nqkv_aux_read_stream: %d" % rc)
    return checksums


def copy(dst: torch.Tensor, src: torch.Tensor, stream=None) -> None:
    assert src.is_contiguous() and dst.is_contiguous() and src.numel() * src.element_size() == dst.numel() * dst.element_size()
    rc = lib.nqkv_aux_copy(dst.data_ptr(), src.data_ptr(), src.numel() * src.element_size(), _stream(stream))
    if rc:
        raise RuntimeError("nqkv_aux_copy: %d" % rc)


def empty_launch(stream=None) -> None:
    rc = lib.nqkv_aux_empty_launch(_stream(stream))
    if rc:
        raise RuntimeError("nqkv_aux_empty_launch: %d" % rc)


def mix_stream(src: torch.Tensor, dst: torch.Tensor, reads: int, writes: int, stream=None) -> int:
    """One pass of the plain read : write mix kernel -> bytes moved (read + written)."""
    assert src.is_contiguous() and dst.is_contiguous()
    tiles = ctypes.c_size_t(0)
    rc = lib.nqkv_aux_mix_stream(src.data_ptr(), src.numel() * src.element_size(), dst.data_ptr(),
                                 dst.numel() * dst.element_size(), reads, writes, ctypes.byref(tiles), _stream(stream))
    if rc:
        raise RuntimeError("nqkv_aux_mix_stream: %d" % rc)
    return tiles.value * 4096 * (reads + writes)

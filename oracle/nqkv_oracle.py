"""ctypes/numpy front end of the NQKV CPU oracle -- TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this
module.  It loads `libnqkv_oracle.so` (built from `nqkv_oracle.cpp` next to this
file with plain g++; built on first use if absent) and marshals numpy arrays.  It
imports nothing from the GPU package and the GPU package imports nothing from here.

All fp16 data crosses this boundary as numpy.uint16 bit patterns (or numpy.float16
arrays, which are viewed as uint16 without conversion).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
import threading

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "nqkv_oracle.cpp")
_LIB = os.path.join(_HERE, "libnqkv_oracle.so")
_CXXFLAGS = ["-O2", "-std=c++17", "-ffp-contract=off", "-fPIC", "-shared", "-pthread"]

_lock = threading.Lock()
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with g++ (no fast-math, no FMA contraction)."""
    stale = (not os.path.exists(_LIB)) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC)
    if force or stale:
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["g++", *_CXXFLAGS, "-o", tmp, _SRC])
        os.replace(tmp, _LIB)
    return _LIB


def _load():
    global _lib
    with _lock:
        if _lib is None:
            build()
            lib = ctypes.CDLL(_LIB)
            c = ctypes
            p = c.c_void_p
            lib.oracle_hardware_threads.restype = c.c_int
            lib.oracle_half_to_float.restype = c.c_float
            lib.oracle_half_to_float.argtypes = [c.c_uint16]
            lib.oracle_float_to_half.restype = c.c_uint16
            lib.oracle_float_to_half.argtypes = [c.c_float]
            lib.oracle_codebook.restype = c.c_int
            lib.oracle_codebook.argtypes = [c.c_int, c.c_int, p, p, p]
            lib.oracle_quantize_block.restype = None
            lib.oracle_quantize_block.argtypes = [p, c.c_int, c.c_int, p, p, p]
            lib.oracle_pack_bits.restype = None
            lib.oracle_pack_bits.argtypes = [p, c.c_int64, c.c_int, p]
            lib.oracle_unpack_bits.restype = None
            lib.oracle_unpack_bits.argtypes = [p, c.c_int64, c.c_int, p]
            lib.oracle_quantize_kv.restype = c.c_int
            lib.oracle_quantize_kv.argtypes = [p, c.c_int64, c.c_int64, c.c_int64,
                                               c.c_int, c.c_int, c.c_int, c.c_int64,
                                               c.c_int, c.c_int, p, c.c_int64, c.c_int64,
                                               p, p, c.c_int]
            lib.oracle_quantize_kv_hidden.restype = c.c_int
            lib.oracle_quantize_kv_hidden.argtypes = [p, c.c_int64, c.c_int64, c.c_int64,
                                                      c.c_int, c.c_int, c.c_int, c.c_int64,
                                                      c.c_int, c.c_int, p, c.c_int64, c.c_int64, p, p, c.c_int]
            lib.oracle_dequantize_kv.restype = c.c_int
            lib.oracle_dequantize_kv.argtypes = [p, p, c.c_int, c.c_int, c.c_int, c.c_int, c.c_int, p,
                                                 c.c_int64, c.c_int64, c.c_int64,
                                                 p, c.c_int64, c.c_int64, c.c_int64, c.c_int]
            lib.oracle_attention_f64.restype = None
            lib.oracle_attention_f64.argtypes = [p, p, p, c.c_int64, c.c_int, c.c_double, p]
            lib.oracle_dequantize_slab_f64.restype = None
            lib.oracle_dequantize_slab_f64.argtypes = [p, p, c.c_int, c.c_int, c.c_int, p, c.c_int64, p]
            lib.oracle_decode_attention.restype = c.c_int
            lib.oracle_decode_attention_multi.argtypes = [p, p, p, p, p, c.c_int, c.c_int, c.c_int, c.c_int,
                                                          c.c_int, p, c.c_int64, c.c_int64, c.c_int,
                                                          c.c_float, p, c.c_int]
            lib.oracle_decode_attention_multi.restype = c.c_int
            lib.oracle_decode_attention.argtypes = [p, p, p, p, p, c.c_int, c.c_int, c.c_int, c.c_int,
                                                    c.c_int, p, c.c_int64, c.c_int64, c.c_float,
                                                    p, c.c_int]
            _lib = lib
    return _lib


def _ptr(a: np.ndarray):
    return a.ctypes.data_as(ctypes.c_void_p)


def _as_u16(a) -> np.ndarray:
    a = np.asarray(a)
    if a.dtype == np.float16:
        a = a.view(np.uint16)
    if a.dtype != np.uint16:
        raise TypeError("fp16 data must be numpy float16 or uint16 bit patterns")
    return a


def hardware_threads() -> int:
    return int(_load().oracle_hardware_threads())


def half_to_float(h: int) -> float:
    return float(_load().oracle_half_to_float(int(h)))


def float_to_half(f: float) -> int:
    return int(_load().oracle_float_to_half(float(f)))


def codebook(k: int, variant: int = 0):
    """-> (levels fp64 [L], levels fp32 [L], thresholds fp32 [L-1])."""
    L = 1 << k
    l64 = np.zeros(L, np.float64)
    l32 = np.zeros(L, np.float32)
    t32 = np.zeros(max(L - 1, 1), np.float32)
    rc = _load().oracle_codebook(k, variant, _ptr(l64), _ptr(l32), _ptr(t32))
    if rc != 0:
        raise ValueError("oracle_codebook: bad argument")
    return l64, l32, t32[: L - 1]


def quantize_block(x, k: int, levels32: np.ndarray):
    """One block of fp16 -> (codes uint8 [blk] unpacked, scale uint16 bits)."""
    x = np.ascontiguousarray(_as_u16(x))
    lv = np.ascontiguousarray(levels32, np.float32)
    assert lv.size == 1 << k
    codes = np.zeros(x.size, np.uint8)
    scale = np.zeros(1, np.uint16)
    _load().oracle_quantize_block(_ptr(x), x.size, k, _ptr(lv), _ptr(codes), _ptr(scale))
    return codes, int(scale[0])


def pack_bits(codes, k: int) -> np.ndarray:
    codes = np.ascontiguousarray(codes, np.uint8)
    out = np.zeros((codes.size * k + 7) // 8, np.uint8)
    _load().oracle_pack_bits(_ptr(codes), codes.size, k, _ptr(out))
    return out


def unpack_bits(data, n: int, k: int) -> np.ndarray:
    data = np.ascontiguousarray(data, np.uint8)
    assert data.size * 8 >= n * k
    out = np.zeros(n, np.uint8)
    _load().oracle_unpack_bits(_ptr(data), n, k, _ptr(out))
    return out


def new_cache(B: int, H: int, D: int, k: int, blk: int, cap_tokens: int):
    """Zeroed host cache: (codes uint8 [B,H,cap,D*k/8], scales uint16 [B,H,cap,D/blk])."""
    return (np.zeros((B, H, cap_tokens, D * k // 8), np.uint8),
            np.zeros((B, H, cap_tokens, D // blk), np.uint16))


def quantize_kv(src, k: int, blk: int, levels32, codes: np.ndarray, scales: np.ndarray,
                dst_off: int = 0, n_threads: int = 1) -> None:
    """src fp16 [B,H,n,D] (any B/H/token strides, D contiguous) -> rows [dst_off, dst_off+n) of the cache."""
    src = _as_u16(src)
    B, H, n, D = src.shape
    assert src.strides[3] == 2
    sb, sh, ss = (s // 2 for s in src.strides[:3])
    lv = np.ascontiguousarray(levels32, np.float32)
    assert lv.size == 1 << k
    assert codes.flags.c_contiguous and scales.flags.c_contiguous
    assert codes.shape[:2] == (B, H) and codes.shape[3] == D * k // 8
    cap = codes.shape[2]
    assert scales.shape == (B, H, cap, D // blk)
    rc = _load().oracle_quantize_kv(_ptr(src), sb, sh, ss, B, H, D, n, k, blk, _ptr(lv),
                                    cap, dst_off, _ptr(codes), _ptr(scales), n_threads)
    if rc != 0:
        raise ValueError("oracle_quantize_kv: bad argument")


def quantize_kv_hidden(src, k: int, blk_hidden: int, levels32, codes: np.ndarray, scales: np.ndarray,
                       dst_off: int = 0, n_threads: int = 1) -> None:
    """Blocks of blk_hidden consecutive elements of the token's hidden vector (its H heads side by
    side).  src fp16 [B,H,n,D] as a view with any B/H/token strides (token-major storage is the
    view x.reshape(B,n,H,D).transpose(1,2)) -> rows [dst_off, dst_off+n) of a cache with one
    scale per token-head (scales [B,H,cap,1])."""
    src = _as_u16(src)
    B, H, n, D = src.shape
    assert src.strides[3] == 2
    sb, sh, ss = (s // 2 for s in src.strides[:3])
    lv = np.ascontiguousarray(levels32, np.float32)
    assert lv.size == 1 << k
    assert codes.flags.c_contiguous and scales.flags.c_contiguous
    assert codes.shape[:2] == (B, H) and codes.shape[3] == D * k // 8
    cap = codes.shape[2]
    assert scales.shape == (B, H, cap, 1)
    rc = _load().oracle_quantize_kv_hidden(_ptr(src), sb, sh, ss, B, H, D, n, k, blk_hidden, _ptr(lv),
                                           cap, dst_off, _ptr(codes), _ptr(scales), n_threads)
    if rc != 0:
        raise ValueError("oracle_quantize_kv_hidden: bad argument")


def dequantize_kv(codes: np.ndarray, scales: np.ndarray, k: int, blk: int, levels32,
                  off: int, n_tokens: int, n_threads: int = 1) -> np.ndarray:
    """-> fp16 bit patterns uint16 [B,H,n_tokens,D]."""
    B, H, cap, row_bytes = codes.shape
    D = row_bytes * 8 // k
    lv = np.ascontiguousarray(levels32, np.float32)
    out = np.zeros((B, H, n_tokens, D), np.uint16)
    rc = _load().oracle_dequantize_kv(_ptr(codes), _ptr(scales), B, H, D, k, blk, _ptr(lv),
                                      cap, off, n_tokens, _ptr(out),
                                      H * n_tokens * D, n_tokens * D, D, n_threads)
    if rc != 0:
        raise ValueError("oracle_dequantize_kv: bad argument")
    return out


def attention_f64(q, K, V, sigma: float = 1.0) -> np.ndarray:
    """Plain fp64 softmax attention of one query row: q [D], K [S,D], V [S,D] -> [D]."""
    q = np.ascontiguousarray(q, np.float64)
    K = np.ascontiguousarray(K, np.float64)
    V = np.ascontiguousarray(V, np.float64)
    S, D = K.shape
    assert V.shape == (S, D) and q.shape == (D,)
    out = np.zeros(D, np.float64)
    _load().oracle_attention_f64(_ptr(q), _ptr(K), _ptr(V), S, D, float(sigma), _ptr(out))
    return out


def dequantize_slab_f64(codes_slab, scales_slab, k: int, blk: int, levels32) -> np.ndarray:
    """Exact fp64 values level*scale of one (batch, head) slab: codes [n, D*k/8] -> [n, D]."""
    codes_slab = np.ascontiguousarray(codes_slab, np.uint8)
    scales_slab = np.ascontiguousarray(_as_u16(scales_slab))
    n, row_bytes = codes_slab.shape
    D = row_bytes * 8 // k
    lv = np.ascontiguousarray(levels32, np.float32)
    X = np.zeros((n, D), np.float64)
    _load().oracle_dequantize_slab_f64(_ptr(codes_slab), _ptr(scales_slab), D, k, blk, _ptr(lv), n, _ptr(X))
    return X


def decode_attention(q, k_codes, k_scales, v_codes, v_scales, k: int, blk: int, levels32,
                     seq_len: int, softmax_scale: float = 1.0, n_threads: int = 1) -> np.ndarray:
    """q fp16 [B,H,D]; caches as in new_cache -> out fp64 [B,H,D]."""
    q = np.ascontiguousarray(_as_u16(q))
    B, H, D = q.shape
    cap = k_codes.shape[2]
    for a in (k_codes, k_scales, v_codes, v_scales):
        assert a.flags.c_contiguous
    assert k_codes.shape == v_codes.shape == (B, H, cap, D * k // 8)
    assert k_scales.shape == v_scales.shape == (B, H, cap, D // blk)
    lv = np.ascontiguousarray(levels32, np.float32)
    out = np.zeros((B, H, D), np.float64)
    rc = _load().oracle_decode_attention(_ptr(q), _ptr(k_codes), _ptr(_as_u16(k_scales)),
                                         _ptr(v_codes), _ptr(_as_u16(v_scales)),
                                         B, H, D, k, blk, _ptr(lv), cap, seq_len,
                                         float(softmax_scale), _ptr(out), n_threads)
    if rc != 0:
        raise ValueError("oracle_decode_attention: bad argument")
    return out


def decode_attention_multi(q, k_codes, k_scales, v_codes, v_scales, k: int, blk: int, levels32,
                           seq_len: int, softmax_scale: float = 1.0, n_threads: int = 1) -> np.ndarray:
    """q fp16 [B,H,Q,D], the queries of the last Q of the first seq_len cached tokens -> fp64 [B,H,Q,D]."""
    q = np.ascontiguousarray(_as_u16(q))
    B, H, Q, D = q.shape
    cap = k_codes.shape[2]
    for a in (k_codes, k_scales, v_codes, v_scales):
        assert a.flags.c_contiguous
    assert k_codes.shape == v_codes.shape == (B, H, cap, D * k // 8)
    assert k_scales.shape == v_scales.shape == (B, H, cap, D // blk)
    lv = np.ascontiguousarray(levels32, np.float32)
    out = np.zeros((B, H, Q, D), np.float64)
    rc = _load().oracle_decode_attention_multi(_ptr(q), _ptr(k_codes), _ptr(_as_u16(k_scales)),
                                               _ptr(v_codes), _ptr(_as_u16(v_scales)),
                                               B, H, D, k, blk, _ptr(lv), cap, seq_len, Q,
                                               float(softmax_scale), _ptr(out), n_threads)
    if rc != 0:
        raise ValueError("oracle_decode_attention_multi: bad argument")
    return out

"""Thin ctypes binding of libnqkv (include/nqkv.h): argument marshalling only.

Every step of the path -- code search, bit packing, table look-up, attention -- runs in the
library's HIP kernels.  torch is used for device memory and the stream handle, nothing else.
Importing this module loads `libnqkv.so` from the package directory and raises if it is not
there: there is no CPU fallback.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np
import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libnqkv.so")

OK, EINVAL, EUNSUPPORTED, EWORKSPACE, EHIP = 0, -1, -2, -3, -4

EXPORTS = ("nqkv_strerror", "nqkv_version", "nqkv_build_codebook",
           "nqkv_quantize_kv", "nqkv_quantize_kv_pair", "nqkv_dequantize_kv",
           "nqkv_decode_workspace_bytes", "nqkv_decode_attention", "nqkv_decode_step",
           "nqkv_decode_attention_static", "nqkv_decode_workspace_init", "nqkv_decode_workspace_check",
           "nqkv_quantize_kv_hidden",
           "nqkv_decode_multi_workspace_bytes", "nqkv_decode_attention_multi", "nqkv_decode_attention_multi_varlen",
           "nqkv_decode_multi_paged_workspace_bytes", "nqkv_decode_attention_multi_paged",
           "nqkv_quantize_kv_pair_varlen", "nqkv_quantize_kv_paged_varlen",
           "nqkv_decode_attention_varlen", "nqkv_decode_step_varlen",
           "nqkv_decode_paged_workspace_bytes", "nqkv_decode_attention_paged", "nqkv_decode_step_paged",
           "nqkv_quantize_kv_paged")


class CacheDesc(ctypes.Structure):
    """Mirror of nqkv_cache_desc."""
    _fields_ = [("B", ctypes.c_int32), ("H", ctypes.c_int32), ("D", ctypes.c_int32),
                ("k", ctypes.c_int32), ("block", ctypes.c_int32), ("flags", ctypes.c_int32),
                ("cap_tokens", ctypes.c_int64)]


class NqkvError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (%d)" % (where, strerror(status), status))


def _load(path: str = LIB_PATH) -> ctypes.CDLL:
    if not os.path.exists(path):
        raise ImportError("%s is not built: run `python -c 'import __graft_entry__ as g; g.build()'` "
                          "(or python paper_2505_16210_amd/build.py) first; there is no fallback path" % os.path.basename(path))
    lib = ctypes.CDLL(path)
    c = ctypes
    vp, i64, i32 = c.c_void_p, c.c_int64, c.c_int
    dp = c.POINTER(CacheDesc)
    fp = c.POINTER(c.c_float)
    lib.nqkv_strerror.restype = c.c_char_p
    lib.nqkv_strerror.argtypes = [i32]
    lib.nqkv_version.restype = i32
    lib.nqkv_build_codebook.restype = i32
    lib.nqkv_build_codebook.argtypes = [i32, i32, fp]
    lib.nqkv_quantize_kv.restype = i32
    lib.nqkv_quantize_kv.argtypes = [dp, fp, vp, i64, i64, i64, i64, i64, vp, vp, vp]
    lib.nqkv_quantize_kv_pair.restype = i32
    lib.nqkv_quantize_kv_pair.argtypes = [dp, fp, vp, vp, i64, i64, i64, i64, i64, vp, vp, vp, vp, vp]
    lib.nqkv_quantize_kv_pair_varlen.restype = i32
    lib.nqkv_quantize_kv_pair_varlen.argtypes = [dp, fp, vp, vp, i64, i64, i64, i64, vp, i64, vp, vp, vp, vp, vp]
    lib.nqkv_quantize_kv_paged_varlen.restype = i32
    lib.nqkv_quantize_kv_paged_varlen.argtypes = [dp, fp, vp, vp, i64, i64, i64, i64, vp, i64, vp, i64, i64,
                                                  vp, vp, vp, vp, vp]
    lib.nqkv_dequantize_kv.restype = i32
    lib.nqkv_dequantize_kv.argtypes = [dp, fp, vp, vp, i64, i64, vp, i64, i64, i64, vp]
    lib.nqkv_decode_workspace_bytes.restype = i32
    lib.nqkv_decode_workspace_bytes.argtypes = [dp, i64, i32, c.POINTER(c.c_size_t), c.POINTER(i32)]
    lib.nqkv_decode_multi_workspace_bytes.restype = i32
    lib.nqkv_decode_multi_workspace_bytes.argtypes = [dp, i64, i32, i32, c.POINTER(c.c_size_t), c.POINTER(i32)]
    lib.nqkv_decode_attention_multi.restype = i32
    lib.nqkv_decode_attention_multi.argtypes = [dp, fp, vp, vp, vp, vp, vp, i64, i32, c.c_float, vp, vp,
                                                c.c_size_t, i32, vp]
    lib.nqkv_decode_attention_multi_varlen.restype = i32
    lib.nqkv_decode_attention_multi_varlen.argtypes = [dp, fp, vp, vp, vp, vp, vp, vp, i64, i32, c.c_float, vp, vp,
                                                       c.c_size_t, i32, vp]
    lib.nqkv_decode_multi_paged_workspace_bytes.restype = i32
    lib.nqkv_decode_multi_paged_workspace_bytes.argtypes = [dp, i64, i32, i32, c.POINTER(c.c_size_t), c.POINTER(i32)]
    lib.nqkv_decode_attention_multi_paged.restype = i32
    lib.nqkv_decode_attention_multi_paged.argtypes = [dp, fp, vp, vp, vp, vp, vp, vp, i64, i64, vp, i64, i32, c.c_float,
                                                      vp, vp, c.c_size_t, i32, vp]
    lib.nqkv_decode_attention.restype = i32
    lib.nqkv_decode_attention.argtypes = [dp, fp, vp, vp, vp, vp, vp, i64, c.c_float, vp, vp,
                                          c.c_size_t, i32, vp]
    lib.nqkv_decode_attention_static.restype = i32
    lib.nqkv_decode_attention_static.argtypes = [dp, fp, vp, vp, vp, vp, vp, i64, c.c_float, vp, i32, vp]
    lib.nqkv_decode_workspace_init.restype = i32
    lib.nqkv_decode_workspace_init.argtypes = [vp, c.c_size_t, vp]
    lib.nqkv_decode_workspace_check.restype = i32
    lib.nqkv_decode_workspace_check.argtypes = [vp, c.c_size_t, vp]
    lib.nqkv_decode_step.restype = i32
    lib.nqkv_decode_step.argtypes = [dp, fp, vp, vp, vp, i64, i64, vp, vp, vp, vp, i64, c.c_float, vp, vp,
                                     c.c_size_t, i32, vp]
    lib.nqkv_decode_attention_varlen.restype = i32
    lib.nqkv_decode_attention_varlen.argtypes = [dp, fp, vp, vp, vp, vp, vp, vp, i64, c.c_float, vp, vp,
                                                 c.c_size_t, i32, vp]
    lib.nqkv_decode_step_varlen.restype = i32
    lib.nqkv_decode_step_varlen.argtypes = [dp, fp, vp, vp, vp, i64, i64, vp, vp, vp, vp, vp, i64, c.c_float, vp, vp,
                                            c.c_size_t, i32, vp]
    lib.nqkv_quantize_kv_paged.restype = i32
    lib.nqkv_quantize_kv_paged.argtypes = [dp, fp, vp, vp, i64, i64, i64, i64, i64, vp, i64, i64, vp, vp, vp, vp, vp]
    lib.nqkv_decode_paged_workspace_bytes.restype = i32
    lib.nqkv_decode_paged_workspace_bytes.argtypes = [dp, i64, c.POINTER(c.c_size_t), c.POINTER(i32)]
    lib.nqkv_decode_attention_paged.restype = i32
    lib.nqkv_decode_attention_paged.argtypes = [dp, fp, vp, vp, vp, vp, vp, vp, i64, i64, vp, i64, c.c_float, vp, vp,
                                                c.c_size_t, vp]
    lib.nqkv_decode_step_paged.restype = i32
    lib.nqkv_decode_step_paged.argtypes = [dp, fp, vp, vp, vp, i64, i64, vp, vp, vp, vp, vp, i64, i64, vp, i64,
                                           c.c_float, vp, vp, c.c_size_t, vp]
    lib.nqkv_quantize_kv_hidden.restype = i32
    lib.nqkv_quantize_kv_hidden.argtypes = [dp, fp, vp, vp, i64, i64, i64, i64, i64, i32, vp, vp, vp, vp, vp]
    return lib


lib = _load()


def use_library(path: str) -> None:
    """Point the binding at another build of the same C ABI (the timestamp-instrumented measurement
    build of build.py --timeline); every later call goes there."""
    global lib
    lib = _load(path)


def strerror(status: int) -> str:
    return lib.nqkv_strerror(int(status)).decode()


def version() -> int:
    return int(lib.nqkv_version())


def _check(rc: int, where: str) -> None:
    if rc != OK:
        raise NqkvError(rc, where)


def _levels_ptr(levels):
    lv = np.ascontiguousarray(levels, dtype=np.float32)
    return lv, lv.ctypes.data_as(ctypes.POINTER(ctypes.c_float))


def _stream(stream) -> int:
    if stream is None:
        stream = torch.cuda.current_stream()
    return stream.cuda_stream if hasattr(stream, "cuda_stream") else int(stream)


def _temp_workspace(need: int, device, stream, zero: bool):
    """A workspace for one call when the caller passed none: allocated (and zero-filled, where the
    kernel expects zeroed counters) ON THE STREAM THE KERNEL WILL RUN ON, so that the fill is
    ordered before the kernel, and recorded on that stream so that the allocator does not hand the
    memory to someone else while the kernel may still be running.  A raw stream handle gives the
    binding nothing to order the fill against: such callers pass their own workspace."""
    if not need:
        return None
    if stream is None:
        stream = torch.cuda.current_stream()
    if not isinstance(stream, torch.cuda.Stream):
        raise ValueError("pass an explicit workspace when launching on a raw stream handle")
    with torch.cuda.stream(stream):
        ws = (torch.zeros if zero else torch.empty)(need, dtype=torch.uint8, device=device)
    ws.record_stream(stream)
    return ws


def _dev_ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def build_codebook(k: int, variant: int = 0) -> np.ndarray:
    """nqkv_build_codebook -> numpy float32 [2^k] (host)."""
    out = np.zeros(1 << max(int(k), 0) if 0 <= int(k) <= 8 else 1, np.float32)
    rc = lib.nqkv_build_codebook(int(k), int(variant), out.ctypes.data_as(ctypes.POINTER(ctypes.c_float)))
    _check(rc, "nqkv_build_codebook")
    return out


FLAG_SCAN_QUANTIZER, FLAG_WORKGROUP_PER_ITEM = 1, 2


def make_desc(B: int, H: int, D: int, k: int, block: int, cap_tokens: int, flags: int = 0) -> CacheDesc:
    return CacheDesc(B, H, D, k, block, flags, cap_tokens)


def alloc_cache(desc: CacheDesc, device="cuda"):
    """Device buffers of the documented layout: (codes uint8 [B,H,cap,D*k/8], scales fp16 [B,H,cap,D/block])."""
    codes = torch.zeros(desc.B, desc.H, desc.cap_tokens, desc.D * desc.k // 8, dtype=torch.uint8, device=device)
    scales = torch.zeros(desc.B, desc.H, desc.cap_tokens, desc.D // desc.block, dtype=torch.float16, device=device)
    return codes, scales


def _src_strides(x: torch.Tensor):
    assert x.dtype == torch.float16 and x.dim() == 4 and x.stride(3) == 1
    return x.stride(0), x.stride(1), x.stride(2)


def quantize_kv(desc: CacheDesc, levels, src: torch.Tensor, codes: torch.Tensor, scales: torch.Tensor,
                dst_token_offset: int = 0, stream=None) -> None:
    """nqkv_quantize_kv: src fp16 [B,H,n,D] (D contiguous) -> cache rows [off, off+n)."""
    lv, lvp = _levels_ptr(levels)
    sb, sh, st = _src_strides(src)
    rc = lib.nqkv_quantize_kv(ctypes.byref(desc), lvp, _dev_ptr(src), sb, sh, st, src.shape[2],
                              dst_token_offset, _dev_ptr(codes), _dev_ptr(scales), _stream(stream))
    _check(rc, "nqkv_quantize_kv")


def quantize_kv_pair(desc: CacheDesc, levels, k_src: torch.Tensor, v_src: torch.Tensor,
                     k_codes, k_scales, v_codes, v_scales, dst_token_offset: int = 0, stream=None) -> None:
    """nqkv_quantize_kv_pair: K and V of equal shape and strides in one launch."""
    lv, lvp = _levels_ptr(levels)
    sb, sh, st = _src_strides(k_src)
    assert _src_strides(v_src) == (sb, sh, st) and v_src.shape == k_src.shape
    rc = lib.nqkv_quantize_kv_pair(ctypes.byref(desc), lvp, _dev_ptr(k_src), _dev_ptr(v_src), sb, sh, st,
                                   k_src.shape[2], dst_token_offset, _dev_ptr(k_codes), _dev_ptr(k_scales),
                                   _dev_ptr(v_codes), _dev_ptr(v_scales), _stream(stream))
    _check(rc, "nqkv_quantize_kv_pair")


def quantize_kv_pair_varlen(desc: CacheDesc, levels, k_src: torch.Tensor, v_src: torch.Tensor,
                            k_codes, k_scales, v_codes, v_scales, dst_token_offsets: torch.Tensor, max_offset: int,
                            stream=None) -> None:
    """nqkv_quantize_kv_pair_varlen: sequence b's tokens go to rows [offsets[b], offsets[b] + n)."""
    lv, lvp = _levels_ptr(levels)
    sb, sh, st = _src_strides(k_src)
    assert _src_strides(v_src) == (sb, sh, st) and v_src.shape == k_src.shape
    rc = lib.nqkv_quantize_kv_pair_varlen(ctypes.byref(desc), lvp, _dev_ptr(k_src), _dev_ptr(v_src), sb, sh, st,
                                          k_src.shape[2], _lens_arg(dst_token_offsets, desc.B), max_offset,
                                          _dev_ptr(k_codes), _dev_ptr(k_scales), _dev_ptr(v_codes), _dev_ptr(v_scales),
                                          _stream(stream))
    _check(rc, "nqkv_quantize_kv_pair_varlen")


def quantize_kv_hidden(desc: CacheDesc, levels, k_src: torch.Tensor, v_src, k_codes, k_scales, v_codes, v_scales,
                       dst_token_offset: int = 0, block_hidden: int = 256, stream=None) -> None:
    """nqkv_quantize_kv_hidden: k_src (and v_src or None) fp16 [B,H,n,D] views, e.g. token-major
    storage x.view(B,n,H,D).transpose(1,2); the cache has one scale per token-head."""
    lv, lvp = _levels_ptr(levels)
    assert k_src.dtype == torch.float16 and k_src.dim() == 4 and (k_src.numel() == 0 or k_src.stride(3) == 1)
    if v_src is not None:
        assert v_src.dtype == torch.float16 and v_src.shape == k_src.shape and v_src.stride() == k_src.stride()
    sb, sh, st = _src_strides(k_src)
    rc = lib.nqkv_quantize_kv_hidden(ctypes.byref(desc), lvp, _dev_ptr(k_src), _dev_ptr(v_src), sb, sh, st,
                                     k_src.shape[2], dst_token_offset, block_hidden,
                                     _dev_ptr(k_codes), _dev_ptr(k_scales), _dev_ptr(v_codes), _dev_ptr(v_scales),
                                     _stream(stream))
    _check(rc, "nqkv_quantize_kv_hidden")


def dequantize_kv(desc: CacheDesc, levels, codes, scales, token_offset: int, n_tokens: int,
                  out: torch.Tensor | None = None, stream=None) -> torch.Tensor:
    """nqkv_dequantize_kv -> fp16 [B,H,n_tokens,D]."""
    lv, lvp = _levels_ptr(levels)
    if out is None:
        out = torch.empty(desc.B, desc.H, n_tokens, desc.D, dtype=torch.float16, device=codes.device)
    sb, sh, st = _src_strides(out)
    rc = lib.nqkv_dequantize_kv(ctypes.byref(desc), lvp, _dev_ptr(codes), _dev_ptr(scales), token_offset,
                                n_tokens, _dev_ptr(out), sb, sh, st, _stream(stream))
    _check(rc, "nqkv_dequantize_kv")
    return out


def decode_workspace_bytes(desc: CacheDesc, seq_len: int, num_splits: int = 0):
    """nqkv_decode_workspace_bytes -> (bytes, splits)."""
    nbytes = ctypes.c_size_t(0)
    splits = ctypes.c_int(0)
    rc = lib.nqkv_decode_workspace_bytes(ctypes.byref(desc), seq_len, num_splits,
                                         ctypes.byref(nbytes), ctypes.byref(splits))
    _check(rc, "nqkv_decode_workspace_bytes")
    return int(nbytes.value), int(splits.value)


def decode_attention(desc: CacheDesc, levels, q: torch.Tensor, k_codes, k_scales, v_codes, v_scales,
                     seq_len: int, softmax_scale: float = 1.0, out: torch.Tensor | None = None,
                     workspace: torch.Tensor | None = None, num_splits: int = 0, stream=None) -> torch.Tensor:
    """nqkv_decode_attention: q fp16 [B,H,D] -> out fp16 [B,H,D]."""
    lv, lvp = _levels_ptr(levels)
    assert q.dtype == torch.float16 and q.is_contiguous()
    if out is None:
        out = torch.empty_like(q)
    ws_bytes = 0
    if workspace is None:
        need, _ = decode_workspace_bytes(desc, seq_len, num_splits)
        workspace = _temp_workspace(need, q.device, stream, zero=True)      # counters start at zero
    if workspace is not None:
        ws_bytes = workspace.numel() * workspace.element_size()
    rc = lib.nqkv_decode_attention(ctypes.byref(desc), lvp, _dev_ptr(q), _dev_ptr(k_codes), _dev_ptr(k_scales),
                                   _dev_ptr(v_codes), _dev_ptr(v_scales), seq_len, float(softmax_scale),
                                   _dev_ptr(out), _dev_ptr(workspace), ws_bytes, num_splits, _stream(stream))
    _check(rc, "nqkv_decode_attention")
    return out


def decode_workspace_init(workspace: torch.Tensor, stream=None) -> None:
    """nqkv_decode_workspace_init: clears the counters of a split-K workspace (on the stream)."""
    rc = lib.nqkv_decode_workspace_init(_dev_ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    _check(rc, "nqkv_decode_workspace_init")


def decode_workspace_check(workspace: torch.Tensor, stream=None) -> int:
    """nqkv_decode_workspace_check -> OK or EWORKSPACE (waits for the stream)."""
    rc = lib.nqkv_decode_workspace_check(_dev_ptr(workspace), workspace.numel() * workspace.element_size(), _stream(stream))
    if rc not in (OK, EWORKSPACE):
        _check(rc, "nqkv_decode_workspace_check")
    return rc


STATIC_SCRATCH_BYTES = 2 << 20


def decode_attention_static(desc: CacheDesc, levels, q: torch.Tensor, k_codes, k_scales, v_codes, v_scales,
                            seq_len: int, softmax_scale: float = 1.0, out: torch.Tensor | None = None,
                            num_splits: int = 0, stream=None) -> torch.Tensor:
    """nqkv_decode_attention_static: as decode_attention, the workspace being the library's own fixed
    array (no allocation inside the call; pass `out` to keep this wrapper from allocating either)."""
    lv, lvp = _levels_ptr(levels)
    assert q.dtype == torch.float16 and q.is_contiguous()
    if out is None:
        out = torch.empty_like(q)
    rc = lib.nqkv_decode_attention_static(ctypes.byref(desc), lvp, _dev_ptr(q), _dev_ptr(k_codes), _dev_ptr(k_scales),
                                          _dev_ptr(v_codes), _dev_ptr(v_scales), seq_len, float(softmax_scale),
                                          _dev_ptr(out), num_splits, _stream(stream))
    _check(rc, "nqkv_decode_attention_static")
    return out


def decode_multi_workspace_bytes(desc: CacheDesc, seq_len: int, q_len: int, num_splits: int = 0):
    """nqkv_decode_multi_workspace_bytes -> (bytes, splits)."""
    nbytes = ctypes.c_size_t(0)
    splits = ctypes.c_int(0)
    rc = lib.nqkv_decode_multi_workspace_bytes(ctypes.byref(desc), seq_len, q_len, num_splits,
                                               ctypes.byref(nbytes), ctypes.byref(splits))
    _check(rc, "nqkv_decode_multi_workspace_bytes")
    return int(nbytes.value), int(splits.value)


def decode_attention_multi(desc: CacheDesc, levels, q: torch.Tensor, k_codes, k_scales, v_codes, v_scales,
                           seq_len: int, softmax_scale: float = 1.0, out: torch.Tensor | None = None,
                           workspace: torch.Tensor | None = None, num_splits: int = 0, stream=None) -> torch.Tensor:
    """nqkv_decode_attention_multi: q fp16 [B,H,Q,D], the queries of the last Q of the first seq_len
    cached tokens -> out fp16 [B,H,Q,D]."""
    lv, lvp = _levels_ptr(levels)
    assert q.dtype == torch.float16 and q.is_contiguous() and q.dim() == 4
    q_len = q.shape[2]
    if out is None:
        out = torch.empty_like(q)
    ws_bytes = 0
    if workspace is None:
        need, _ = decode_multi_workspace_bytes(desc, seq_len, q_len, num_splits)
        workspace = _temp_workspace(need, q.device, stream, zero=False)
    if workspace is not None:
        ws_bytes = workspace.numel() * workspace.element_size()
    rc = lib.nqkv_decode_attention_multi(ctypes.byref(desc), lvp, _dev_ptr(q), _dev_ptr(k_codes), _dev_ptr(k_scales),
                                         _dev_ptr(v_codes), _dev_ptr(v_scales), seq_len, q_len, float(softmax_scale),
                                         _dev_ptr(out), _dev_ptr(workspace), ws_bytes, num_splits, _stream(stream))
    _check(rc, "nqkv_decode_attention_multi")
    return out


def decode_attention_multi_varlen(desc: CacheDesc, levels, q: torch.Tensor, k_codes, k_scales, v_codes, v_scales,
                                  seq_lens: torch.Tensor, max_seq_len: int, softmax_scale: float = 1.0,
                                  out: torch.Tensor | None = None, workspace: torch.Tensor | None = None,
                                  num_splits: int = 0, stream=None) -> torch.Tensor:
    """nqkv_decode_attention_multi_varlen: seq_lens int32 [B] on the device; q fp16 [B,H,Q,D]."""
    lv, lvp = _levels_ptr(levels)
    assert q.dtype == torch.float16 and q.is_contiguous() and q.dim() == 4
    assert seq_lens.dtype == torch.int32 and seq_lens.is_contiguous() and seq_lens.numel() == desc.B
    q_len = q.shape[2]
    if out is None:
        out = torch.empty_like(q)
    ws_bytes = 0
    if workspace is None:
        need, _ = decode_multi_workspace_bytes(desc, max_seq_len, q_len, num_splits)
        workspace = _temp_workspace(need, q.device, stream, zero=False)
    if workspace is not None:
        ws_bytes = workspace.numel() * workspace.element_size()
    rc = lib.nqkv_decode_attention_multi_varlen(ctypes.byref(desc), lvp, _dev_ptr(q), _dev_ptr(k_codes), _dev_ptr(k_scales),
                                                _dev_ptr(v_codes), _dev_ptr(v_scales), _dev_ptr(seq_lens), max_seq_len,
                                                q_len, float(softmax_scale), _dev_ptr(out), _dev_ptr(workspace), ws_bytes,
                                                num_splits, _stream(stream))
    _check(rc, "nqkv_decode_attention_multi_varlen")
    return out


def decode_step(desc: CacheDesc, levels, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                k_codes, k_scales, v_codes, v_scales, pos: int, softmax_scale: float = 1.0,
                out: torch.Tensor | None = None, workspace: torch.Tensor | None = None,
                num_splits: int = 0, stream=None) -> torch.Tensor:
    """nqkv_decode_step: k_new, v_new fp16 [B,H,1,D] or [B,H,D] (D contiguous) -> out fp16 [B,H,D];
    the caches gain row `pos`."""
    lv, lvp = _levels_ptr(levels)
    assert q.dtype == torch.float16 and q.is_contiguous()
    if k_new.dim() == 4:
        k_new, v_new = k_new[:, :, 0], v_new[:, :, 0]
    assert k_new.dtype == torch.float16 and k_new.stride(2) == 1 and k_new.stride() == v_new.stride()
    if out is None:
        out = torch.empty_like(q)
    ws_bytes = 0
    if workspace is None:
        need, _ = decode_workspace_bytes(desc, max(pos, 1), num_splits)
        workspace = _temp_workspace(need, q.device, stream, zero=True)      # counters start at zero
    if workspace is not None:
        ws_bytes = workspace.numel() * workspace.element_size()
    rc = lib.nqkv_decode_step(ctypes.byref(desc), lvp, _dev_ptr(q), _dev_ptr(k_new), _dev_ptr(v_new),
                              k_new.stride(0), k_new.stride(1), _dev_ptr(k_codes), _dev_ptr(k_scales),
                              _dev_ptr(v_codes), _dev_ptr(v_scales), pos, float(softmax_scale), _dev_ptr(out),
                              _dev_ptr(workspace), ws_bytes, num_splits, _stream(stream))
    _check(rc, "nqkv_decode_step")
    return out


def _lens_arg(lens: torch.Tensor, B: int):
    assert lens.dtype == torch.int32 and lens.is_contiguous() and lens.numel() == B and lens.is_cuda
    return _dev_ptr(lens)


def decode_attention_varlen(desc: CacheDesc, levels, q: torch.Tensor, k_codes, k_scales, v_codes, v_scales,
                            seq_lens: torch.Tensor, max_seq_len: int, softmax_scale: float = 1.0,
                            out: torch.Tensor | None = None, workspace: torch.Tensor | None = None,
                            num_splits: int = 0, stream=None) -> torch.Tensor:
    """nqkv_decode_attention_varlen: seq_lens int32 [B] on the device, max_seq_len its host upper bound."""
    lv, lvp = _levels_ptr(levels)
    assert q.dtype == torch.float16 and q.is_contiguous()
    if out is None:
        out = torch.empty_like(q)
    ws_bytes = 0
    if workspace is None:
        need, _ = decode_workspace_bytes(desc, max_seq_len, num_splits)
        workspace = _temp_workspace(need, q.device, stream, zero=True)      # counters start at zero
    if workspace is not None:
        ws_bytes = workspace.numel() * workspace.element_size()
    rc = lib.nqkv_decode_attention_varlen(ctypes.byref(desc), lvp, _dev_ptr(q), _dev_ptr(k_codes), _dev_ptr(k_scales),
                                          _dev_ptr(v_codes), _dev_ptr(v_scales), _lens_arg(seq_lens, desc.B),
                                          max_seq_len, float(softmax_scale), _dev_ptr(out), _dev_ptr(workspace),
                                          ws_bytes, num_splits, _stream(stream))
    _check(rc, "nqkv_decode_attention_varlen")
    return out


def decode_step_varlen(desc: CacheDesc, levels, q: torch.Tensor, k_new: torch.Tensor, v_new: torch.Tensor,
                       k_codes, k_scales, v_codes, v_scales, pos: torch.Tensor, max_pos: int,
                       softmax_scale: float = 1.0, out: torch.Tensor | None = None,
                       workspace: torch.Tensor | None = None, num_splits: int = 0, stream=None) -> torch.Tensor:
    """nqkv_decode_step_varlen: pos int32 [B] on the device (cached rows of each sequence), max_pos its
    host upper bound; the caches gain row pos[b] of every sequence b."""
    lv, lvp = _levels_ptr(levels)
    assert q.dtype == torch.float16 and q.is_contiguous()
    if k_new.dim() == 4:
        k_new, v_new = k_new[:, :, 0], v_new[:, :, 0]
    assert k_new.dtype == torch.float16 and k_new.stride(2) == 1 and k_new.stride() == v_new.stride()
    if out is None:
        out = torch.empty_like(q)
    ws_bytes = 0
    if workspace is None:
        need, _ = decode_workspace_bytes(desc, max(max_pos, 1), num_splits)
        workspace = _temp_workspace(need, q.device, stream, zero=True)      # counters start at zero
    if workspace is not None:
        ws_bytes = workspace.numel() * workspace.element_size()
    rc = lib.nqkv_decode_step_varlen(ctypes.byref(desc), lvp, _dev_ptr(q), _dev_ptr(k_new), _dev_ptr(v_new),
                                     k_new.stride(0), k_new.stride(1), _dev_ptr(k_codes), _dev_ptr(k_scales),
                                     _dev_ptr(v_codes), _dev_ptr(v_scales), _lens_arg(pos, desc.B), max_pos,
                                     float(softmax_scale), _dev_ptr(out), _dev_ptr(workspace), ws_bytes, num_splits,
                                     _stream(stream))
    _check(rc, "nqkv_decode_step_varlen")
    return out


def alloc_paged_pool(desc: CacheDesc, num_pages: int, device="cuda"):
    """Pool of pages for the paged calls (desc.cap_tokens = tokens per page):
    (codes uint8 [num_pages,H,P,D*k/8], scales fp16 [num_pages,H,P,D/block])."""
    P = desc.cap_tokens
    codes = torch.zeros(num_pages, desc.H, P, desc.D * desc.k // 8, dtype=torch.uint8, device=device)
    scales = torch.zeros(num_pages, desc.H, P, desc.D // desc.block, dtype=torch.float16, device=device)
    return codes, scales


def decode_paged_workspace_bytes(desc: CacheDesc, max_tokens: int):
    """nqkv_decode_paged_workspace_bytes -> (bytes, pages per sequence)."""
    nbytes = ctypes.c_size_t(0)
    pages = ctypes.c_int(0)
    rc = lib.nqkv_decode_paged_workspace_bytes(ctypes.byref(desc), max_tokens, ctypes.byref(nbytes), ctypes.byref(pages))
    _check(rc, "nqkv_decode_paged_workspace_bytes")
    return int(nbytes.value), int(pages.value)


def _table_arg(block_table: torch.Tensor, B: int):
    assert block_table.dtype == torch.int32 and block_table.dim() == 2 and block_table.shape[0] == B
    assert block_table.is_cuda and block_table.stride(1) == 1
    return _dev_ptr(block_table), block_table.stride(0)


def quantize_kv_paged(desc: CacheDesc, levels, k_src: torch.Tensor, v_src, k_codes, k_scales, v_codes, v_scales,
                      block_table: torch.Tensor, dst_token_offset: int = 0, stream=None) -> None:
    """nqkv_quantize_kv_paged: k_src (and v_src or None) fp16 [B,H,n,D] -> rows [off, off+n) of every
    sequence, in the pages its block-table row names."""
    lv, lvp = _levels_ptr(levels)
    sb, sh, st = _src_strides(k_src)
    if v_src is not None:
        assert v_src.shape == k_src.shape and v_src.stride() == k_src.stride()
    tp, ts = _table_arg(block_table, desc.B)
    rc = lib.nqkv_quantize_kv_paged(ctypes.byref(desc), lvp, _dev_ptr(k_src), _dev_ptr(v_src), sb, sh, st,
                                    k_src.shape[2], dst_token_offset, tp, ts, k_codes.shape[0],
                                    _dev_ptr(k_codes), _dev_ptr(k_scales), _dev_ptr(v_codes), _dev_ptr(v_scales),
                                    _stream(stream))
    _check(rc, "nqkv_quantize_kv_paged")


def quantize_kv_paged_varlen(desc: CacheDesc, levels, k_src: torch.Tensor, v_src, k_codes, k_scales, v_codes, v_scales,
                             block_table: torch.Tensor, dst_token_offsets: torch.Tensor, max_offset: int,
                             stream=None) -> None:
    """nqkv_quantize_kv_paged_varlen: rows [offsets[b], offsets[b] + n) of sequence b, in its pages."""
    lv, lvp = _levels_ptr(levels)
    sb, sh, st = _src_strides(k_src)
    if v_src is not None:
        assert v_src.shape == k_src.shape and v_src.stride() == k_src.stride()
    tp, ts = _table_arg(block_table, desc.B)
    rc = lib.nqkv_quantize_kv_paged_varlen(ctypes.byref(desc), lvp, _dev_ptr(k_src), _dev_ptr(v_src), sb, sh, st,
                                           k_src.shape[2], _lens_arg(dst_token_offsets, desc.B), max_offset,
                                           tp, ts, k_codes.shape[0],
                                           _dev_ptr(k_codes), _dev_ptr(k_scales), _dev_ptr(v_codes), _dev_ptr(v_scales),
                                           _stream(stream))
    _check(rc, "nqkv_quantize_kv_paged_varlen")


def decode_attention_paged(desc: CacheDesc, levels, q, k_codes, k_scales, v_codes, v_scales,
                           block_table: torch.Tensor, seq_lens: torch.Tensor, max_seq_len: int,
                           softmax_scale: float = 1.0, out=None, workspace=None, stream=None) -> torch.Tensor:
    """nqkv_decode_attention_paged: pools [num_pages,H,P,*], block_table int32 [B,max_pages] (device)."""
    lv, lvp = _levels_ptr(levels)
    assert q.dtype == torch.float16 and q.is_contiguous()
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        need, _ = decode_paged_workspace_bytes(desc, max_seq_len)
        workspace = _temp_workspace(need, q.device, stream, zero=True)
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    tp, ts = _table_arg(block_table, desc.B)
    rc = lib.nqkv_decode_attention_paged(ctypes.byref(desc), lvp, _dev_ptr(q), _dev_ptr(k_codes), _dev_ptr(k_scales),
                                         _dev_ptr(v_codes), _dev_ptr(v_scales), tp, ts, k_codes.shape[0],
                                         _lens_arg(seq_lens, desc.B), max_seq_len, float(softmax_scale), _dev_ptr(out),
                                         _dev_ptr(workspace), ws_bytes, _stream(stream))
    _check(rc, "nqkv_decode_attention_paged")
    return out


def decode_multi_paged_workspace_bytes(desc: CacheDesc, max_seq_len: int, q_len: int, num_splits: int = 0):
    """nqkv_decode_multi_paged_workspace_bytes -> (bytes, splits)."""
    nbytes = ctypes.c_size_t(0)
    splits = ctypes.c_int(0)
    rc = lib.nqkv_decode_multi_paged_workspace_bytes(ctypes.byref(desc), max_seq_len, q_len, num_splits,
                                                     ctypes.byref(nbytes), ctypes.byref(splits))
    _check(rc, "nqkv_decode_multi_paged_workspace_bytes")
    return int(nbytes.value), int(splits.value)


def decode_attention_multi_paged(desc: CacheDesc, levels, q, k_codes, k_scales, v_codes, v_scales,
                                 block_table: torch.Tensor, seq_lens: torch.Tensor, max_seq_len: int,
                                 softmax_scale: float = 1.0, out=None, workspace=None, num_splits: int = 0,
                                 stream=None) -> torch.Tensor:
    """nqkv_decode_attention_multi_paged: pools [num_pages,H,P,*], block_table int32 [B,max_pages], q fp16 [B,H,Q,D]."""
    lv, lvp = _levels_ptr(levels)
    assert q.dtype == torch.float16 and q.is_contiguous() and q.dim() == 4
    q_len = q.shape[2]
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        need, _ = decode_multi_paged_workspace_bytes(desc, max_seq_len, q_len, num_splits)
        workspace = _temp_workspace(need, q.device, stream, zero=False)
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    tp, ts = _table_arg(block_table, desc.B)
    rc = lib.nqkv_decode_attention_multi_paged(ctypes.byref(desc), lvp, _dev_ptr(q), _dev_ptr(k_codes), _dev_ptr(k_scales),
                                               _dev_ptr(v_codes), _dev_ptr(v_scales), tp, ts, k_codes.shape[0],
                                               _lens_arg(seq_lens, desc.B), max_seq_len, q_len, float(softmax_scale),
                                               _dev_ptr(out), _dev_ptr(workspace), ws_bytes, num_splits, _stream(stream))
    _check(rc, "nqkv_decode_attention_multi_paged")
    return out


def decode_step_paged(desc: CacheDesc, levels, q, k_new, v_new, k_codes, k_scales, v_codes, v_scales,
                      block_table: torch.Tensor, pos: torch.Tensor, max_pos: int, softmax_scale: float = 1.0,
                      out=None, workspace=None, stream=None) -> torch.Tensor:
    """nqkv_decode_step_paged: appends row pos[b] of every sequence into its page and attends."""
    lv, lvp = _levels_ptr(levels)
    assert q.dtype == torch.float16 and q.is_contiguous()
    if k_new.dim() == 4:
        k_new, v_new = k_new[:, :, 0], v_new[:, :, 0]
    assert k_new.dtype == torch.float16 and k_new.stride(2) == 1 and k_new.stride() == v_new.stride()
    if out is None:
        out = torch.empty_like(q)
    if workspace is None:
        need, _ = decode_paged_workspace_bytes(desc, max(max_pos, 1))
        workspace = _temp_workspace(need, q.device, stream, zero=True)
    ws_bytes = workspace.numel() * workspace.element_size() if workspace is not None else 0
    tp, ts = _table_arg(block_table, desc.B)
    rc = lib.nqkv_decode_step_paged(ctypes.byref(desc), lvp, _dev_ptr(q), _dev_ptr(k_new), _dev_ptr(v_new),
                                    k_new.stride(0), k_new.stride(1), _dev_ptr(k_codes), _dev_ptr(k_scales),
                                    _dev_ptr(v_codes), _dev_ptr(v_scales), tp, ts, k_codes.shape[0],
                                    _lens_arg(pos, desc.B), max_pos, float(softmax_scale), _dev_ptr(out),
                                    _dev_ptr(workspace), ws_bytes, _stream(stream))
    _check(rc, "nqkv_decode_step_paged")
    return out

"""Thin ctypes binding of libkvq.so: the same names as include/kvq.h, argument marshalling only.

PyTorch is used for device memory and streams; every step of the path runs in the library's
kernels.  Loading fails loudly when the library has not been built.
"""
from __future__ import annotations

import ctypes
import os
from typing import Optional

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvq.so")

KVQ_OK, KVQ_ERR_INVALID_ARG, KVQ_ERR_UNSUPPORTED, KVQ_ERR_CAPACITY, KVQ_ERR_HIP = range(5)
KVQ_BF16, KVQ_FP32 = 0, 1
KVQ_META_FP32, KVQ_META_FP8_BF16 = 0, 1
KVQ_KEYS_PER_TOKEN, KVQ_KEYS_PER_CHANNEL = 0, 1

# Every symbol declared in include/kvq.h.
EXPORTED = (
    "kvq_cache_bytes", "kvq_cache_create", "kvq_cache_destroy", "kvq_cache_len", "kvq_cache_reset",
    "kvq_cache_truncate", "kvq_cache_evict", "kvq_cache_set_rotation_signs", "kvq_quantize_append",
    "kvq_quantize_append_static", "kvq_chunk_attention", "kvq_chunk_attention_fp32",
    "kvq_chunk_attention_ex", "kvq_attention_diagnostics",
    "kvq_cache_export", "kvq_status_string", "kvq_version",
)


class kvq_cache_desc(ctypes.Structure):
    _fields_ = [("num_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32), ("bits", ctypes.c_int32),
                ("group_size", ctypes.c_int32), ("rotate", ctypes.c_int32), ("io_dtype", ctypes.c_int32),
                ("meta_format", ctypes.c_int32), ("key_axis", ctypes.c_int32), ("capacity_tokens", ctypes.c_int64)]


class kvq_attention_opts(ctypes.Structure):
    _fields_ = [("q_heads_per_kv_head", ctypes.c_int32), ("causal", ctypes.c_int32),
                ("q_stride_token", ctypes.c_int64), ("q_stride_head", ctypes.c_int64)]


class KvqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__("%s: %s (status %d)" % (where, kvq_status_string(status), status))


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise ImportError("libkvq.so is not built: run `python -m paper_2605_26266_amd.build` "
                          "(or __graft_entry__.build()) first; there is no fallback path")
    L = ctypes.CDLL(LIB_PATH)
    vp, i64, ci, cf = ctypes.c_void_p, ctypes.c_int64, ctypes.c_int, ctypes.c_float
    dp = ctypes.POINTER(kvq_cache_desc)
    L.kvq_cache_bytes.argtypes = [dp]
    L.kvq_cache_bytes.restype = ctypes.c_size_t
    L.kvq_cache_create.argtypes = [dp, vp, ctypes.c_size_t, ctypes.POINTER(vp)]
    L.kvq_cache_destroy.argtypes = [vp]
    L.kvq_cache_destroy.restype = None
    L.kvq_cache_len.argtypes = [vp]
    L.kvq_cache_len.restype = i64
    L.kvq_cache_reset.argtypes = [vp]
    L.kvq_cache_truncate.argtypes = [vp, i64]
    L.kvq_cache_evict.argtypes = [vp, i64]
    L.kvq_cache_set_rotation_signs.argtypes = [vp, ctypes.c_char_p]
    L.kvq_quantize_append.argtypes = [vp, vp, vp, i64, i64, i64, vp]
    L.kvq_quantize_append_static.argtypes = [vp, vp, vp, i64, i64, i64, vp]
    att = [vp, i64, i64, vp, vp, vp, i64, i64, i64, i64, cf, ci, vp, vp, vp]
    L.kvq_chunk_attention.argtypes = att
    L.kvq_chunk_attention_fp32.argtypes = att
    L.kvq_chunk_attention_ex.argtypes = att[:12] + [ctypes.POINTER(kvq_attention_opts)] + att[12:]
    L.kvq_attention_diagnostics.argtypes = [vp, i64, i64, vp, vp, vp, vp, vp, i64, i64, i64, i64, cf, ci, vp, vp]
    L.kvq_cache_export.argtypes = [vp, ci, i64, i64, vp, vp, vp, vp]
    L.kvq_status_string.argtypes = [ci]
    L.kvq_status_string.restype = ctypes.c_char_p
    L.kvq_version.restype = ctypes.c_char_p
    _lib = L
    return L


def kvq_status_string(status: int) -> str:
    return lib().kvq_status_string(int(status)).decode()


def kvq_version() -> str:
    return lib().kvq_version().decode()


def _check(status: int, where: str) -> None:
    if status != KVQ_OK:
        raise KvqError(status, where)


def _stream(stream: Optional[torch.cuda.Stream]) -> int:
    s = torch.cuda.current_stream() if stream is None else stream
    return int(s.cuda_stream)


def _ptr(t: Optional[torch.Tensor]) -> Optional[int]:
    return None if t is None else t.data_ptr()


def make_desc(num_heads: int, head_dim: int, bits: int, capacity_tokens: int, io_dtype: int = KVQ_BF16,
              group_size: Optional[int] = None, rotate: int = 1, meta_format: int = KVQ_META_FP32,
              key_axis: int = KVQ_KEYS_PER_TOKEN) -> kvq_cache_desc:
    return kvq_cache_desc(num_heads, head_dim, bits, head_dim if group_size is None else group_size, rotate,
                          io_dtype, meta_format, key_axis, capacity_tokens)


def kvq_cache_bytes(desc: kvq_cache_desc) -> int:
    return int(lib().kvq_cache_bytes(ctypes.byref(desc)))


class Cache:
    """Owner of the device storage (a torch uint8 tensor) and of the host-side kvq_cache handle."""

    def __init__(self, desc: kvq_cache_desc, device: str = "cuda:0"):
        self.desc = desc
        nbytes = kvq_cache_bytes(desc)
        if nbytes == 0:
            _check(kvq_cache_create_status(desc), "kvq_cache_create")
        self.storage = torch.empty(nbytes, dtype=torch.uint8, device=device)
        handle = ctypes.c_void_p()
        _check(lib().kvq_cache_create(ctypes.byref(desc), self.storage.data_ptr(), nbytes, ctypes.byref(handle)),
               "kvq_cache_create")
        self.handle = handle
        self.torch_dtype = torch.bfloat16 if desc.io_dtype == KVQ_BF16 else torch.float32

    def __len__(self) -> int:
        return int(lib().kvq_cache_len(self.handle))

    def close(self) -> None:
        if getattr(self, "handle", None):
            lib().kvq_cache_destroy(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass


def kvq_cache_create_status(desc: kvq_cache_desc) -> int:
    """Status that kvq_cache_create returns for this description without any storage (validation only)."""
    handle = ctypes.c_void_p()
    return int(lib().kvq_cache_create(ctypes.byref(desc), None, 0, ctypes.byref(handle)))


def kvq_cache_len(cache: Cache) -> int:
    return len(cache)


def kvq_cache_reset(cache: Cache) -> None:
    _check(lib().kvq_cache_reset(cache.handle), "kvq_cache_reset")


def kvq_cache_truncate(cache: Cache, new_len: int) -> None:
    _check(lib().kvq_cache_truncate(cache.handle, int(new_len)), "kvq_cache_truncate")


def kvq_cache_evict(cache: Cache, n_tokens: int) -> None:
    _check(lib().kvq_cache_evict(cache.handle, int(n_tokens)), "kvq_cache_evict")


def kvq_cache_set_rotation_signs(cache: Cache, negate) -> None:
    """negate: None or a sequence of head_dim truthy/falsy entries (truthy = sign -1)."""
    buf = None
    if negate is not None:
        flags = bytes(1 if x else 0 for x in negate)
        if len(flags) != cache.desc.head_dim:
            raise ValueError("negate must have head_dim entries")
        buf = flags
    _check(lib().kvq_cache_set_rotation_signs(cache.handle, buf), "kvq_cache_set_rotation_signs")


def _tok_head_strides(t: torch.Tensor):
    if t.dim() != 3 or t.stride(2) != 1:
        raise ValueError("expected a [token][head][channel] tensor with unit channel stride")
    return t.stride(0), t.stride(1)


def _check_shape(t: Optional[torch.Tensor], heads: int, head_dim: int, what: str, tokens: Optional[int] = None) -> None:
    """The kernels index [token][head][channel] by the cache's head count and head_dim: a tensor with fewer heads
    or channels would be read or written out of bounds on the device, so the shape is checked here."""
    if t is None:
        return
    if t.dim() != 3 or t.shape[1] != heads or t.shape[2] != head_dim or (tokens is not None and t.shape[0] != tokens):
        raise ValueError("%s must be [%s][%d][%d], got %s" % (what, "tokens" if tokens is None else tokens, heads,
                                                              head_dim, tuple(t.shape)))


def kvq_quantize_append(cache: Cache, k: torch.Tensor, v: torch.Tensor,
                        stream: Optional[torch.cuda.Stream] = None) -> None:
    if k.dtype != cache.torch_dtype or v.dtype != cache.torch_dtype or k.shape != v.shape:
        raise ValueError("k and v must share the cache's io dtype and one shape")
    _check_shape(k, cache.desc.num_heads, cache.desc.head_dim, "k and v")
    st, sh = _tok_head_strides(k)
    if _tok_head_strides(v) != (st, sh):
        raise ValueError("k and v must share strides")
    _check(lib().kvq_quantize_append(cache.handle, k.data_ptr(), v.data_ptr(), k.shape[0], st, sh, _stream(stream)),
           "kvq_quantize_append")


def kvq_quantize_append_static(cache: Cache, k: torch.Tensor, v: torch.Tensor,
                               stream: Optional[torch.cuda.Stream] = None) -> None:
    """kvq_quantize_append with the per-channel work space in the library's static device array."""
    if k.dtype != cache.torch_dtype or v.dtype != cache.torch_dtype or k.shape != v.shape:
        raise ValueError("k and v must share the cache's io dtype and one shape")
    _check_shape(k, cache.desc.num_heads, cache.desc.head_dim, "k and v")
    st, sh = _tok_head_strides(k)
    if _tok_head_strides(v) != (st, sh):
        raise ValueError("k and v must share strides")
    _check(lib().kvq_quantize_append_static(cache.handle, k.data_ptr(), v.data_ptr(), k.shape[0], st, sh,
                                            _stream(stream)), "kvq_quantize_append_static")


def _attention(fn, cache: Cache, cache_start: int, cache_len: int, q, k_cur, v_cur, softmax_scale, correction,
               out, mass_cached, stream):
    st, sh = _tok_head_strides(q)
    n_cur = 0 if k_cur is None else k_cur.shape[0]
    H, d = cache.desc.num_heads, cache.desc.head_dim
    _check_shape(q, H, d, "q")
    _check_shape(out, H, d, "out", q.shape[0])
    _check_shape(k_cur, H, d, "k_cur")
    _check_shape(v_cur, H, d, "v_cur", n_cur)
    if mass_cached is not None and mass_cached.numel() != H * q.shape[0]:
        raise ValueError("mass_cached must hold heads * m values")
    for t in (k_cur, v_cur, out):
        if t is not None and (t.dtype != cache.torch_dtype or (t.shape[0] > 0 and _tok_head_strides(t) != (st, sh))):
            raise ValueError("q, k_cur, v_cur and out must share dtype and strides")
    if q.dtype != cache.torch_dtype:
        raise ValueError("q must be in the cache's io dtype")
    if mass_cached is not None and (mass_cached.dtype != torch.float32 or not mass_cached.is_contiguous()):
        raise ValueError("mass_cached must be a contiguous float32 [heads][m] tensor")
    _check(fn(cache.handle, int(cache_start), int(cache_len), q.data_ptr(), _ptr(k_cur), _ptr(v_cur), q.shape[0],
              n_cur, st, sh, float(softmax_scale), int(correction), out.data_ptr(), _ptr(mass_cached),
              _stream(stream)), "kvq_chunk_attention")


def kvq_chunk_attention(cache: Cache, cache_start: int, cache_len: int, q: torch.Tensor,
                        k_cur: Optional[torch.Tensor], v_cur: Optional[torch.Tensor], out: torch.Tensor,
                        mass_cached: Optional[torch.Tensor] = None, softmax_scale: float = 0.0,
                        correction: int = 1, stream: Optional[torch.cuda.Stream] = None) -> None:
    _attention(lib().kvq_chunk_attention, cache, cache_start, cache_len, q, k_cur, v_cur, softmax_scale, correction,
               out, mass_cached, stream)


def kvq_chunk_attention_ex(cache: Cache, cache_start: int, cache_len: int, q: torch.Tensor,
                           k_cur: Optional[torch.Tensor], v_cur: Optional[torch.Tensor], out: torch.Tensor,
                           mass_cached: Optional[torch.Tensor] = None, softmax_scale: float = 0.0,
                           correction: int = 1, causal: bool = False,
                           stream: Optional[torch.cuda.Stream] = None) -> None:
    """Grouped-query heads (q has a multiple of the cache's head count) and / or a causal current block."""
    kv = k_cur if k_cur is not None else v_cur
    if q.shape[1] % cache.desc.num_heads != 0:
        raise ValueError("query heads must be a multiple of the cache's heads")
    for t in (k_cur, v_cur):
        if t is not None and (t.dtype != cache.torch_dtype or (kv.shape[0] > 0 and _tok_head_strides(t) != _tok_head_strides(kv))):
            raise ValueError("k_cur and v_cur must share dtype and strides")
    if q.dtype != cache.torch_dtype or out.dtype != cache.torch_dtype or _tok_head_strides(out) != _tok_head_strides(q):
        raise ValueError("q and out must be in the cache's io dtype and share strides")
    if mass_cached is not None and (mass_cached.dtype != torch.float32 or not mass_cached.is_contiguous()):
        raise ValueError("mass_cached must be a contiguous float32 [query heads][m] tensor")
    n_cur_tokens = 0 if k_cur is None else k_cur.shape[0]
    _check_shape(q, q.shape[1], cache.desc.head_dim, "q")
    _check_shape(out, q.shape[1], cache.desc.head_dim, "out", q.shape[0])
    _check_shape(k_cur, cache.desc.num_heads, cache.desc.head_dim, "k_cur")
    _check_shape(v_cur, cache.desc.num_heads, cache.desc.head_dim, "v_cur", n_cur_tokens)
    if mass_cached is not None and mass_cached.numel() != q.shape[1] * q.shape[0]:
        raise ValueError("mass_cached must hold query heads * m values")
    qst, qsh = _tok_head_strides(q)
    st, sh = _tok_head_strides(kv) if kv is not None and kv.shape[0] > 0 else (cache.desc.num_heads * cache.desc.head_dim, cache.desc.head_dim)
    opts = kvq_attention_opts(q.shape[1] // cache.desc.num_heads, int(bool(causal)), qst, qsh)
    n_cur = 0 if k_cur is None else k_cur.shape[0]
    _check(lib().kvq_chunk_attention_ex(cache.handle, int(cache_start), int(cache_len), q.data_ptr(), _ptr(k_cur),
                                        _ptr(v_cur), q.shape[0], n_cur, st, sh, float(softmax_scale), int(correction),
                                        ctypes.byref(opts), out.data_ptr(), _ptr(mass_cached), _stream(stream)),
           "kvq_chunk_attention_ex")


def kvq_attention_diagnostics(cache: Cache, cache_start: int, cache_len: int, q: torch.Tensor,
                              k_ref: Optional[torch.Tensor], v_ref: Optional[torch.Tensor],
                              k_cur: Optional[torch.Tensor], v_cur: Optional[torch.Tensor], diag: torch.Tensor,
                              softmax_scale: float = 0.0, correction: int = 1,
                              stream: Optional[torch.cuda.Stream] = None) -> None:
    """diag: float32 [heads][m][4] = (P_S unquantized, P_S quantized, JSD in nats, output MSE) per row.
    k_ref / v_ref: the unquantized tokens of the window [cache_len][heads][d]; all [token][head][d]
    tensors must share dtype and strides."""
    tensors = [t for t in (k_ref, v_ref, k_cur, v_cur) if t is not None and t.shape[0] > 0]
    if q.dtype != cache.torch_dtype or any(t.dtype != cache.torch_dtype for t in tensors):
        raise ValueError("tensors must be in the cache's io dtype")
    if len({_tok_head_strides(t) for t in tensors + [q]}) > 1:
        raise ValueError("q, k_ref, v_ref, k_cur and v_cur must share strides")
    if k_ref is not None and (k_ref.shape[0] != cache_len or v_ref is None or v_ref.shape[0] != cache_len):
        raise ValueError("k_ref and v_ref must hold cache_len tokens")
    if diag.dtype != torch.float32 or not diag.is_contiguous() or diag.numel() != cache.desc.num_heads * q.shape[0] * 4:
        raise ValueError("diag must be a contiguous float32 [heads][m][4] tensor")
    for t, what in ((q, "q"), (k_ref, "k_ref"), (v_ref, "v_ref"), (k_cur, "k_cur"), (v_cur, "v_cur")):
        _check_shape(t, cache.desc.num_heads, cache.desc.head_dim, what)
    st, sh = _tok_head_strides(q)
    n_cur = 0 if k_cur is None else k_cur.shape[0]
    _check(lib().kvq_attention_diagnostics(cache.handle, int(cache_start), int(cache_len), q.data_ptr(), _ptr(k_ref),
                                           _ptr(v_ref), _ptr(k_cur), _ptr(v_cur), q.shape[0], n_cur, st, sh,
                                           float(softmax_scale), int(correction), diag.data_ptr(), _stream(stream)),
           "kvq_attention_diagnostics")


def kvq_chunk_attention_fp32(cache: Cache, cache_start: int, cache_len: int, q: torch.Tensor,
                             k_cur: Optional[torch.Tensor], v_cur: Optional[torch.Tensor], out: torch.Tensor,
                             mass_cached: Optional[torch.Tensor] = None, softmax_scale: float = 0.0,
                             correction: int = 1, stream: Optional[torch.cuda.Stream] = None) -> None:
    _attention(lib().kvq_chunk_attention_fp32, cache, cache_start, cache_len, q, k_cur, v_cur, softmax_scale,
               correction, out, mass_cached, stream)


def kvq_cache_export(cache: Cache, which: int, start: int, count: int, codes: Optional[torch.Tensor],
                     scales: Optional[torch.Tensor], zeros: Optional[torch.Tensor],
                     stream: Optional[torch.cuda.Stream] = None) -> None:
    _check(lib().kvq_cache_export(cache.handle, int(which), int(start), int(count), _ptr(codes), _ptr(scales),
                                  _ptr(zeros), _stream(stream)), "kvq_cache_export")


def export_all(cache: Cache, which: int, start: int = 0, count: Optional[int] = None):
    """Allocate outputs and export: (codes uint8 [H][count][d], scales, zeros); scales and zeros are
    [H][count] for per-token caches and [H][count][G] for KVQ_META_FP8_BF16 caches."""
    count = len(cache) - start if count is None else count
    H, d = cache.desc.num_heads, cache.desc.head_dim
    dev = cache.storage.device
    codes = torch.empty((H, count, d), dtype=torch.uint8, device=dev)
    meta_shape = (H, count) if cache.desc.meta_format == KVQ_META_FP32 else (H, count, d // cache.desc.group_size)
    if which == 0 and cache.desc.key_axis == KVQ_KEYS_PER_CHANNEL:
        meta_shape = (H, count, d)   # every token carries the per-channel values of its block
    scales = torch.empty(meta_shape, dtype=torch.float32, device=dev)
    zeros = torch.empty(meta_shape, dtype=torch.float32, device=dev)
    kvq_cache_export(cache, which, start, count, codes, scales, zeros)
    return codes, scales, zeros

"""Thin Python binding of libkvq's C ABI (include/kvq.h): argument marshalling only.

Every step of the path runs in the HIP kernels of libkvq.so; torch is used for device memory
and streams.  There is no fallback: if the library is missing the import of the functions
below raises.
"""
from __future__ import annotations

import ctypes as C
import functools
import os
from dataclasses import dataclass

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libkvq.so")

KVQ_F16, KVQ_BF16, KVQ_F32 = 0, 1, 2
AXIS_HEAD_DIM, AXIS_SEQ = 0, 1
OK, ERR_INVALID_ARG, ERR_UNSUPPORTED, ERR_CAPACITY, ERR_WORKSPACE, ERR_DEVICE, ERR_STATIC_SCRATCH = range(7)
STATIC_SCRATCH_BYTES = 4 << 20

_DTYPES = {torch.float16: KVQ_F16, torch.bfloat16: KVQ_BF16, torch.float32: KVQ_F32}


class KvqError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {status_string(status)} (status {status})")


class _CLayout(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("batch", "kv_heads", "max_seq", "head_dim", "bits_k", "bits_v", "group_k",
                                          "group_v", "axis_k", "axis_v", "raw_dtype", "rotate_k")] + [("signs_k", C.c_uint32 * 4), ("rotate_v", C.c_int32), ("signs_v", C.c_uint32 * 4),
                                                                       ("page_tokens", C.c_int32), ("n_pages", C.c_int32),
                                                                       ("resid_len", C.c_int32)]


class _CCache(C.Structure):
    _fields_ = [(n, C.c_void_p) for n in ("k_codes", "k_meta", "v_codes", "v_meta", "k_resid", "v_resid", "page_table",
                                          "v_scale_exp")]


_lib = None


def load():
    """Loads libkvq.so (built by `paper_2502_15075_amd.build`); raises if it is not there."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError(f"{LIB_PATH} is missing: run `python -m paper_2502_15075_amd.build` (there is no fallback path)")
        lib = C.CDLL(LIB_PATH)
        lib.kvq_cache_bytes.argtypes = [C.POINTER(_CLayout), C.POINTER(C.c_size_t)]
        lib.kvq_residual_bytes.argtypes = [C.POINTER(_CLayout), C.POINTER(C.c_size_t)]
        lib.kvq_decode_workspace_bytes.argtypes = [C.POINTER(_CLayout), C.c_int32, C.c_int32, C.POINTER(C.c_size_t)]
        lib.kvq_quantize_append.argtypes = [C.POINTER(_CLayout), C.POINTER(_CCache), C.c_void_p, C.c_void_p, C.c_int,
                                            C.c_int64, C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.c_void_p]
        lib.kvq_decode_attention.argtypes = [C.POINTER(_CLayout), C.POINTER(_CCache), C.c_void_p, C.c_int, C.c_int32,
                                             C.c_int32, C.c_float, C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]
        lib.kvq_decode_attention_static.argtypes = [C.POINTER(_CLayout), C.POINTER(_CCache), C.c_void_p, C.c_int, C.c_int32,
                                                    C.c_int32, C.c_float, C.c_void_p, C.c_int, C.c_void_p]
        lib.kvq_decode_step.argtypes = [C.POINTER(_CLayout), C.POINTER(_CCache), C.c_void_p, C.c_void_p, C.c_int, C.c_int64,
                                        C.c_int64, C.c_int32, C.c_void_p, C.c_int, C.c_int32, C.c_float, C.c_void_p, C.c_int,
                                        C.c_void_p, C.c_size_t, C.c_void_p]
        lib.kvq_decode_attention_varlen.argtypes = [C.POINTER(_CLayout), C.POINTER(_CCache), C.c_void_p, C.c_int, C.c_int32,
                                                    C.c_void_p, C.c_int32, C.c_float, C.c_void_p, C.c_int, C.c_void_p,
                                                    C.c_size_t, C.c_void_p]
        lib.kvq_decode_step_varlen.argtypes = [C.POINTER(_CLayout), C.POINTER(_CCache), C.c_void_p, C.c_void_p, C.c_int,
                                               C.c_int64, C.c_int64, C.c_void_p, C.c_int32, C.c_void_p, C.c_int, C.c_int32,
                                               C.c_float, C.c_void_p, C.c_int, C.c_void_p, C.c_size_t, C.c_void_p]
        lib.kvq_dequantize.argtypes = [C.POINTER(_CLayout), C.POINTER(_CCache), C.c_int32, C.c_int32, C.c_void_p,
                                       C.c_void_p, C.c_int, C.c_void_p]
        lib.kvq_reconstruction_error.argtypes = [C.POINTER(_CLayout), C.POINTER(_CCache), C.c_void_p, C.c_void_p, C.c_int,
                                                 C.c_int64, C.c_int64, C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p]
        lib.kvq_selftest_quantizer.argtypes = [C.c_void_p, C.c_void_p]
        lib.kvq_status_string.argtypes = [C.c_int]
        lib.kvq_status_string.restype = C.c_char_p
        for f in ("kvq_cache_bytes", "kvq_residual_bytes", "kvq_decode_workspace_bytes", "kvq_quantize_append", "kvq_decode_attention",
                  "kvq_decode_step", "kvq_dequantize", "kvq_reconstruction_error", "kvq_decode_attention_varlen",
                  "kvq_decode_step_varlen", "kvq_selftest_quantizer", "kvq_decode_attention_static"):
            getattr(lib, f).restype = C.c_int
        _lib = lib
    return _lib


def status_string(status: int) -> str:
    return load().kvq_status_string(int(status)).decode()


@dataclass(frozen=True)
class Layout:
    """Mirror of kvq_layout."""
    batch: int
    kv_heads: int
    max_seq: int
    head_dim: int = 128
    bits_k: int = 4
    bits_v: int = 2
    group_k: int = 64
    group_v: int = 64
    axis_k: int = AXIS_HEAD_DIM
    axis_v: int = AXIS_HEAD_DIM
    raw_dtype: int = KVQ_F16
    rotate_k: int = 0
    signs_k: tuple = (0, 0, 0, 0)
    rotate_v: int = 0
    signs_v: tuple = (0, 0, 0, 0)
    page_tokens: int = 0
    n_pages: int = 0
    resid_len: int = 0

    def c(self) -> _CLayout:
        st = self.__dict__.get("_c")                         # (kept on the object: hashing 18 fields per call costs 1.5 us)
        if st is None:
            st = _layout_struct(self)
            object.__setattr__(self, "_c", st)
        return st


@functools.lru_cache(maxsize=256)
def _layout_struct(L: Layout) -> _CLayout:
    """The C struct of a layout, built once per distinct layout (the library only reads it)."""
    return _CLayout(L.batch, L.kv_heads, L.max_seq, L.head_dim, L.bits_k, L.bits_v, L.group_k, L.group_v, L.axis_k, L.axis_v,
                    L.raw_dtype, L.rotate_k, (C.c_uint32 * 4)(*L.signs_k), L.rotate_v, (C.c_uint32 * 4)(*L.signs_v),
                    L.page_tokens, L.n_pages, L.resid_len)


def _check(status: int, where: str) -> None:
    if status != OK:
        raise KvqError(status, where)


def _stream_ptr():
    # (the raw handle of torch's current stream: the same value as torch.cuda.current_stream().cuda_stream, without
    # building a Stream object per call)
    return C.c_void_p(torch._C._cuda_getCurrentRawStream(torch.cuda.current_device()))


def _p(t):
    return C.c_void_p(0 if t is None else t.data_ptr())


def cache_bytes(layout: Layout):
    out = (C.c_size_t * 4)()
    cl = layout.c()
    _check(load().kvq_cache_bytes(C.byref(cl), out), "kvq_cache_bytes")
    return [int(v) for v in out]


def residual_bytes(layout: Layout):
    out = (C.c_size_t * 2)()
    cl = layout.c()
    _check(load().kvq_residual_bytes(C.byref(cl), out), "kvq_residual_bytes")
    return [int(v) for v in out]


def decode_workspace_bytes(layout: Layout, q_heads: int, seq_len: int) -> int:
    out = C.c_size_t()
    cl = layout.c()
    _check(load().kvq_decode_workspace_bytes(C.byref(cl), q_heads, seq_len, C.byref(out)), "kvq_decode_workspace_bytes")
    return int(out.value)


class Cache:
    """The caller-owned device planes (torch uint8 tensors) of one layer: codes and scale/zero of keys and values,
    then the two residual buffers of channel-wise keys (None otherwise)."""

    def __init__(self, layout: Layout, device="cuda", fill=None):
        self.layout = layout
        sizes = cache_bytes(layout) + residual_bytes(layout)
        mk = (lambda n: torch.empty(n, dtype=torch.uint8, device=device)) if fill is None else \
             (lambda n: torch.full((n,), fill, dtype=torch.uint8, device=device))
        self.planes = [mk(n) if n else None for n in sizes]
        # per (batch, kv head): largest exponent field of the value scales of 64 and more stored so far; starts at zero
        self.v_scale_exp = torch.zeros(layout.batch * layout.kv_heads, dtype=torch.int32, device=device)

    # int32 device tensor [B, pages per sequence] of a paged cache (None otherwise); setting it rebuilds the C struct
    @property
    def page_table(self):
        return self.__dict__.get("_page_table")

    @page_table.setter
    def page_table(self, table):
        self.__dict__["_page_table"] = table
        self.__dict__["_struct"] = None

    def c(self) -> _CCache:
        st = self.__dict__.get("_struct")
        if st is None:                                      # the planes never move: the struct is built once per table
            table = self.page_table
            st = self._struct = _CCache(*[(0 if p is None else p.data_ptr()) for p in self.planes],
                                        0 if table is None else table.data_ptr(), self.v_scale_exp.data_ptr())
        return st

    def batch_element(self, b: int, layout: "Layout") -> "Cache":
        """A view of batch element b's share of every plane as a cache of batch 1 (`layout`: this cache's layout with
        batch = 1; contiguous planes only)."""
        assert layout.batch == 1 and layout.page_tokens == 0 and self.layout.page_tokens == 0
        B = self.layout.batch
        sub = Cache.__new__(Cache)
        sub.layout = layout
        sub.planes = [None if p is None else p.view(B, -1)[b] for p in self.planes]
        sub.v_scale_exp = self.v_scale_exp.view(B, -1)[b]
        return sub

    def nbytes(self) -> int:
        return sum(0 if p is None else p.numel() for p in self.planes)


def quantize_append(layout: Layout, cache: Cache, k_new: torch.Tensor, v_new: torch.Tensor, pos: int) -> None:
    """k_new, v_new: [B, H_kv, n_new, D] fp16/bf16 device tensors, last axis contiguous."""
    assert k_new.shape == v_new.shape and k_new.dtype == v_new.dtype and k_new.dim() == 4
    assert k_new.stride() == v_new.stride() and k_new.stride(3) == 1
    cl, cc = layout.c(), cache.c()
    st = load().kvq_quantize_append(C.byref(cl), C.byref(cc), _p(k_new), _p(v_new), _DTYPES[k_new.dtype],
                                    k_new.stride(0), k_new.stride(1), k_new.stride(2), pos, k_new.shape[2], _stream_ptr())
    _check(st, "kvq_quantize_append")


def decode_attention(layout: Layout, cache: Cache, q: torch.Tensor, seq_len: int, softmax_scale: float,
                     out: torch.Tensor, workspace: torch.Tensor) -> torch.Tensor:
    """q: [B, H_q, D] contiguous fp16/bf16; out: [B, H_q, D] contiguous fp32/fp16/bf16; workspace: uint8 device tensor."""
    assert q.is_contiguous() and out.is_contiguous() and q.dim() == 3 and out.shape == q.shape
    cl, cc = layout.c(), cache.c()
    st = load().kvq_decode_attention(C.byref(cl), C.byref(cc), _p(q), _DTYPES[q.dtype], q.shape[1], seq_len,
                                     C.c_float(softmax_scale), _p(out), _DTYPES[out.dtype], _p(workspace),
                                     0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_ptr())
    _check(st, "kvq_decode_attention")
    return out


def decode_attention_static(layout: Layout, cache: Cache, q: torch.Tensor, seq_len: int, softmax_scale: float,
                            out: torch.Tensor) -> torch.Tensor:
    """decode_attention without a workspace argument: the partial records go to the library's static device array
    (at most STATIC_SCRATCH_BYTES of them; calls that overlap on one GPU race on it)."""
    assert q.is_contiguous() and out.is_contiguous() and q.dim() == 3 and out.shape == q.shape
    cl, cc = layout.c(), cache.c()
    st = load().kvq_decode_attention_static(C.byref(cl), C.byref(cc), _p(q), _DTYPES[q.dtype], q.shape[1], seq_len,
                                            C.c_float(softmax_scale), _p(out), _DTYPES[out.dtype], _stream_ptr())
    _check(st, "kvq_decode_attention_static")
    return out


def decode_step(layout: Layout, cache: Cache, k_new: torch.Tensor, v_new: torch.Tensor, pos: int, q: torch.Tensor,
                softmax_scale: float, out: torch.Tensor, workspace) -> torch.Tensor:
    """Fused step: quantize the new token (k_new, v_new: [B, H_kv, D] or [B, H_kv, 1, D]) into position pos, then attend
    over [0, pos].  q, out, workspace as in decode_attention (workspace may be None when no bytes are needed)."""
    if k_new.dim() == 4:
        k_new, v_new = k_new[:, :, 0], v_new[:, :, 0]
    assert k_new.shape == v_new.shape and k_new.dtype == v_new.dtype and k_new.dim() == 3
    assert k_new.stride() == v_new.stride() and k_new.stride(2) == 1
    assert q.is_contiguous() and out.is_contiguous() and q.dim() == 3 and out.shape == q.shape
    cl, cc = layout.c(), cache.c()
    st = load().kvq_decode_step(C.byref(cl), C.byref(cc), _p(k_new), _p(v_new), _DTYPES[k_new.dtype], k_new.stride(0),
                                k_new.stride(1), pos, _p(q), _DTYPES[q.dtype], q.shape[1], C.c_float(softmax_scale), _p(out),
                                _DTYPES[out.dtype], _p(workspace),
                                0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_ptr())
    _check(st, "kvq_decode_step")
    return out


def dequantize(layout: Layout, cache: Cache, t0: int, t1: int, k_out, v_out) -> None:
    """k_out, v_out: [B, H_kv, t1-t0, D] contiguous (fp32/fp16/bf16) or None."""
    ref = k_out if k_out is not None else v_out
    for t in (k_out, v_out):
        assert t is None or (t.is_contiguous() and t.dtype == ref.dtype)
    cl, cc = layout.c(), cache.c()
    st = load().kvq_dequantize(C.byref(cl), C.byref(cc), t0, t1, _p(k_out), _p(v_out), _DTYPES[ref.dtype], _stream_ptr())
    _check(st, "kvq_dequantize")


def reconstruction_error(layout: Layout, cache: Cache, k_ref, v_ref, t0: int, sums: torch.Tensor) -> torch.Tensor:
    """k_ref, v_ref: [B, H_kv, n, D] fp16/bf16 rows of tokens [t0, t0+n) (last axis contiguous; either may be None);
    sums: [B, H_kv, 2] float64 device tensor, overwritten with the squared error of keys and of values per head."""
    ref = k_ref if k_ref is not None else v_ref
    for t in (k_ref, v_ref):
        assert t is None or (t.dim() == 4 and t.dtype == ref.dtype and t.stride() == ref.stride() and t.stride(3) == 1)
    assert sums.dtype == torch.float64 and sums.is_contiguous() and sums.numel() == layout.batch * layout.kv_heads * 2
    cl, cc = layout.c(), cache.c()
    st = load().kvq_reconstruction_error(C.byref(cl), C.byref(cc), _p(k_ref), _p(v_ref), _DTYPES[ref.dtype], ref.stride(0),
                                         ref.stride(1), ref.stride(2), t0, t0 + ref.shape[2], _p(sums), _stream_ptr())
    _check(st, "kvq_reconstruction_error")
    return sums


def selftest_quantizer(counters: torch.Tensor) -> torch.Tensor:
    """counters: int32/uint32 device tensor of 2 elements, overwritten with the numbers of scales and of sampled quotients
    whose fast division differs from IEEE division on this device (both must be 0)."""
    assert counters.numel() == 2 and counters.element_size() == 4 and counters.is_contiguous()
    _check(load().kvq_selftest_quantizer(_p(counters), _stream_ptr()), "kvq_selftest_quantizer")
    return counters


def decode_attention_varlen(layout: Layout, cache: Cache, q: torch.Tensor, seq_lens: torch.Tensor, max_seq_len: int,
                            softmax_scale: float, out: torch.Tensor, workspace) -> torch.Tensor:
    """As decode_attention with one length per batch element: seq_lens is an int32 device tensor [B], max_seq_len an
    upper bound of its values (the workspace is sized for it)."""
    assert q.is_contiguous() and out.is_contiguous() and q.dim() == 3 and out.shape == q.shape
    assert seq_lens.dtype == torch.int32 and seq_lens.is_contiguous() and seq_lens.numel() == layout.batch
    cl, cc = layout.c(), cache.c()
    st = load().kvq_decode_attention_varlen(C.byref(cl), C.byref(cc), _p(q), _DTYPES[q.dtype], q.shape[1], _p(seq_lens),
                                            max_seq_len, C.c_float(softmax_scale), _p(out), _DTYPES[out.dtype], _p(workspace),
                                            0 if workspace is None else workspace.numel() * workspace.element_size(),
                                            _stream_ptr())
    _check(st, "kvq_decode_attention_varlen")
    return out


def decode_step_varlen(layout: Layout, cache: Cache, k_new: torch.Tensor, v_new: torch.Tensor, pos: torch.Tensor,
                       max_pos: int, q: torch.Tensor, softmax_scale: float, out: torch.Tensor, workspace) -> torch.Tensor:
    """As decode_step with one position per batch element: pos is an int32 device tensor [B], max_pos its upper bound."""
    if k_new.dim() == 4:
        assert k_new.shape[2] == 1
        k_new, v_new = k_new[:, :, 0], v_new[:, :, 0]
    assert k_new.shape == v_new.shape and k_new.stride() == v_new.stride() and k_new.stride(2) == 1
    assert q.is_contiguous() and out.is_contiguous() and out.shape == q.shape
    assert pos.dtype == torch.int32 and pos.is_contiguous() and pos.numel() == layout.batch
    cl, cc = layout.c(), cache.c()
    st = load().kvq_decode_step_varlen(C.byref(cl), C.byref(cc), _p(k_new), _p(v_new), _DTYPES[k_new.dtype], k_new.stride(0),
                                       k_new.stride(1), _p(pos), max_pos, _p(q), _DTYPES[q.dtype], q.shape[1],
                                       C.c_float(softmax_scale), _p(out), _DTYPES[out.dtype], _p(workspace),
                                       0 if workspace is None else workspace.numel() * workspace.element_size(), _stream_ptr())
    _check(st, "kvq_decode_step_varlen")
    return out

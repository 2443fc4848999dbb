"""ctypes view of the C oracle in ``kvq_oracle.c`` (test infrastructure only).

The arithmetic lives in the C file; this module only builds it, marshals numpy arrays and
hands back numpy arrays.  It imports nothing from the GPU package.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass, replace

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "kvq_oracle.c")
_LIB = os.path.join(_HERE, "libkvq_oracle.so")

F16, BF16, F32 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (strict IEEE: no contraction, no fast-math).  KVQ_ORACLE_LIB names a library built
    some other way from the same source (a sanitizer build, say) to load instead."""
    if os.environ.get("KVQ_ORACLE_LIB"):
        return os.environ["KVQ_ORACLE_LIB"]
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fPIC", "-shared", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


class _Layout(C.Structure):
    _fields_ = [(n, C.c_int32) for n in ("batch", "kv_heads", "max_seq", "head_dim", "bits_k", "bits_v",
                                          "group_k", "group_v", "raw_dtype", "rotate_k")] + [("signs_k", C.c_uint32 * 4), ("axis_k", C.c_int32), ("rotate_v", C.c_int32), ("signs_v", C.c_uint32 * 4),
                                                                                          ("resid_len", C.c_int32)]


@dataclass(frozen=True)
class Layout:
    batch: int
    kv_heads: int
    max_seq: int
    head_dim: int = 128
    bits_k: int = 4
    bits_v: int = 2
    group_k: int = 64
    group_v: int = 64
    raw_dtype: int = F16
    rotate_k: int = 0
    signs_k: tuple = (0, 0, 0, 0)      # 128 sign bits, little-endian: bit d set means s_d = -1
    axis_k: int = 0                    # 1: channel-wise key groups (group_k tokens) + residual buffer
    rotate_v: int = 0
    signs_v: tuple = (0, 0, 0, 0)
    resid_len: int = 0                 # slots of the residual buffer: 0 = none (axis_k 0) or group_k (axis_k 1)

    def c(self) -> _Layout:
        return _Layout(self.batch, self.kv_heads, self.max_seq, self.head_dim, self.bits_k, self.bits_v,
                       self.group_k, self.group_v, self.raw_dtype, self.rotate_k, (C.c_uint32 * 4)(*self.signs_k),
                       self.axis_k, self.rotate_v, (C.c_uint32 * 4)(*self.signs_v), self.resid_len)


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.ref_f16_to_f32.restype = C.c_float
        _lib.ref_f16_to_f32.argtypes = [C.c_uint16]
        _lib.ref_f32_to_f16.restype = C.c_uint16
        _lib.ref_f32_to_f16.argtypes = [C.c_float]
        _lib.ref_bf16_to_f32.restype = C.c_float
        _lib.ref_bf16_to_f32.argtypes = [C.c_uint16]
        _lib.ref_reconstruct.restype = C.c_float
        _lib.ref_reconstruct.argtypes = [C.c_uint32, C.c_uint16, C.c_uint16]
        _lib.ref_mse.restype = C.c_double
        _lib.ref_mse.argtypes = [C.c_void_p, C.c_void_p, C.c_int64]
        _lib.ref_quantize_group.restype = None
        _lib.ref_quantize_group.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p, C.c_void_p, C.c_void_p]
    return _lib


def threads() -> int:
    """Threads the oracle's loops over independent (batch, head) streams use (OMP_NUM_THREADS, else every core)."""
    return int(lib().ref_threads())


def _ptr(a):
    return None if a is None else a.ctypes.data_as(C.c_void_p)


def dtype_code(a: np.ndarray, bf16: bool = False) -> int:
    """numpy has no bfloat16: bf16 data travels as uint16 bit patterns with bf16=True."""
    if a.dtype == np.float32:
        return F32
    if a.dtype == np.float16:
        return F16
    if a.dtype == np.uint16:
        return BF16 if bf16 else F16
    raise TypeError(a.dtype)


def f32_to_f16_bits(x) -> np.ndarray:
    x = np.ascontiguousarray(x, dtype=np.float32).ravel()
    f = lib().ref_f32_to_f16
    return np.array([f(float(v)) for v in x], dtype=np.uint16)


def f16_bits_to_f32(h) -> np.ndarray:
    h = np.ascontiguousarray(h, dtype=np.uint16).ravel()
    f = lib().ref_f16_to_f32
    return np.array([f(int(v)) for v in h], dtype=np.float32)


def plane_bytes(L: Layout):
    out = (C.c_uint64 * 4)()
    cl = L.c()
    lib().ref_plane_bytes(C.byref(cl), out)
    return [int(v) for v in out]


def new_planes(L: Layout, fill: int = 0):
    """Four uint8 planes (k_codes, k_meta, v_codes, v_meta) of the sizes the format needs."""
    return [np.full(n, fill, dtype=np.uint8) for n in plane_bytes(L)]


def quantize_group(x: np.ndarray, bits: int):
    """One group -> (codes uint8[n], scale_bits, zero_bits)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    codes = np.zeros(x.size, dtype=np.uint8)
    S = C.c_uint16()
    Z = C.c_uint16()
    lib().ref_quantize_group(_ptr(x), x.size, bits, _ptr(codes), C.byref(S), C.byref(Z))
    return codes, int(S.value), int(Z.value)


def quantize_append(L: Layout, planes, k_new: np.ndarray, v_new: np.ndarray, pos: int, bf16: bool = False) -> None:
    """k_new, v_new: contiguous [B, H, n_new, D] arrays (float16, float32, or uint16 bit patterns)."""
    assert k_new.shape == v_new.shape and k_new.flags.c_contiguous and v_new.flags.c_contiguous
    B, H, n_new, D = k_new.shape
    assert (B, H, D) == (L.batch, L.kv_heads, L.head_dim)
    cl = L.c()
    rc = lib().ref_quantize_append(C.byref(cl), _ptr(planes[0]), _ptr(planes[1]), _ptr(planes[2]), _ptr(planes[3]),
                                   _ptr(k_new), _ptr(v_new), C.c_int(dtype_code(k_new, bf16)),
                                   C.c_int64(H * n_new * D), C.c_int64(n_new * D), C.c_int64(D),
                                   C.c_int32(pos), C.c_int32(n_new))
    if rc:
        raise ValueError(f"ref_quantize_append rc={rc}")


def _signs_array(signs):
    return (C.c_uint32 * 4)(*signs)


def rotate(x: np.ndarray, signs=(0, 0, 0, 0)) -> np.ndarray:
    """R x for one vector (binary32), R = H diag(s) / sqrt(n)."""
    x = np.ascontiguousarray(x, dtype=np.float32)
    y = np.zeros_like(x)
    lib().ref_rotate(_ptr(x), C.c_int(x.size), _signs_array(signs), _ptr(y))
    return y


def unrotate(y: np.ndarray, signs=(0, 0, 0, 0)) -> np.ndarray:
    """R^T y for one vector (binary32)."""
    y = np.ascontiguousarray(y, dtype=np.float32)
    x = np.zeros_like(y)
    lib().ref_unrotate(_ptr(y), C.c_int(y.size), _signs_array(signs), _ptr(x))
    return x


def dequantize(L: Layout, planes, t0: int, t1: int, stored: bool = False):
    """Reconstruction of tokens [t0, t1); stored=True keeps rotated keys in the rotated basis."""
    shape = (L.batch, L.kv_heads, t1 - t0, L.head_dim)
    k = np.zeros(shape, dtype=np.float32)
    v = np.zeros(shape, dtype=np.float32)
    cl = L.c()
    fn = lib().ref_dequantize_stored if stored else lib().ref_dequantize
    rc = fn(C.byref(cl), _ptr(planes[0]), _ptr(planes[1]), _ptr(planes[2]), _ptr(planes[3]),
                              C.c_int32(t0), C.c_int32(t1), _ptr(k), _ptr(v))
    if rc:
        raise ValueError(f"ref_dequantize rc={rc}")
    return k, v


def attention_dense(K: np.ndarray, V: np.ndarray, q: np.ndarray, softmax_scale: float, bf16: bool = False) -> np.ndarray:
    """K, V: float32 [B, H_kv, T, D]; q: [B, H_q, D]; returns float32 [B, H_q, D]."""
    K = np.ascontiguousarray(K, dtype=np.float32)
    V = np.ascontiguousarray(V, dtype=np.float32)
    q = np.ascontiguousarray(q)
    B, Hk, T, D = K.shape
    Hq = q.shape[1]
    out = np.zeros((B, Hq, D), dtype=np.float32)
    rc = lib().ref_attention_dense(_ptr(K), _ptr(V), C.c_int32(B), C.c_int32(Hk), C.c_int32(Hq), C.c_int32(T),
                                   C.c_int32(D), _ptr(q), C.c_int(dtype_code(q, bf16)), C.c_float(softmax_scale), _ptr(out))
    if rc:
        raise ValueError(f"ref_attention_dense rc={rc}")
    return out


def decode_attention(L: Layout, planes, q: np.ndarray, seq_len: int, softmax_scale: float, bf16: bool = False) -> np.ndarray:
    q = np.ascontiguousarray(q)
    Hq = q.shape[1]
    out = np.zeros((L.batch, Hq, L.head_dim), dtype=np.float32)
    cl = L.c()
    rc = lib().ref_decode_attention(C.byref(cl), _ptr(planes[0]), _ptr(planes[1]), _ptr(planes[2]), _ptr(planes[3]),
                                    _ptr(q), C.c_int(dtype_code(q, bf16)), C.c_int32(Hq), C.c_int32(seq_len),
                                    C.c_float(softmax_scale), _ptr(out))
    if rc:
        raise ValueError(f"ref_decode_attention rc={rc}")
    return out


def mse(a: np.ndarray, ahat: np.ndarray) -> float:
    a = np.ascontiguousarray(a, dtype=np.float32)
    ahat = np.ascontiguousarray(ahat, dtype=np.float32)
    return float(lib().ref_mse(_ptr(a), _ptr(ahat), C.c_int64(a.size)))


# ---- channel-wise keys with a residual buffer (axis_k = 1): six planes = the four above + k_resid, v_resid

def new_seq_planes(L: Layout, fill: int = 0):
    out = (C.c_uint64 * 2)()
    cl = L.c()
    lib().ref_resid_bytes(C.byref(cl), out)
    return new_planes(L, fill) + [np.full(int(n), fill, dtype=np.uint8) for n in out]


def seq_append(L: Layout, planes, k_new: np.ndarray, v_new: np.ndarray, pos: int, bf16: bool = False) -> None:
    """k_new, v_new: contiguous [B, H, n_new, D] 16-bit arrays (float16, or uint16 patterns); pos = tokens so far."""
    assert k_new.shape == v_new.shape and k_new.flags.c_contiguous and v_new.flags.c_contiguous
    B, H, n_new, D = k_new.shape
    cl = L.c()
    rc = lib().ref_seq_append(C.byref(cl), *[_ptr(p) for p in planes], _ptr(k_new), _ptr(v_new),
                              C.c_int(dtype_code(k_new, bf16)), C.c_int64(H * n_new * D), C.c_int64(n_new * D), C.c_int64(D),
                              C.c_int32(pos), C.c_int32(n_new))
    if rc:
        raise ValueError(f"ref_seq_append rc={rc}")


def seq_dequantize(L: Layout, planes, seq_len: int, t0: int, t1: int):
    shape = (L.batch, L.kv_heads, t1 - t0, L.head_dim)
    k = np.zeros(shape, dtype=np.float32)
    v = np.zeros(shape, dtype=np.float32)
    cl = L.c()
    rc = lib().ref_seq_dequantize(C.byref(cl), *[_ptr(p) for p in planes], C.c_int32(seq_len), C.c_int32(t0), C.c_int32(t1),
                                  _ptr(k), _ptr(v))
    if rc:
        raise ValueError(f"ref_seq_dequantize rc={rc}")
    return k, v


def seq_decode_attention(L: Layout, planes, q: np.ndarray, seq_len: int, softmax_scale: float, bf16: bool = False) -> np.ndarray:
    q = np.ascontiguousarray(q)
    out = np.zeros(q.shape, dtype=np.float32)
    cl = L.c()
    rc = lib().ref_seq_decode_attention(C.byref(cl), *[_ptr(p) for p in planes], _ptr(q), C.c_int(dtype_code(q, bf16)),
                                        C.c_int32(q.shape[1]), C.c_int32(seq_len), C.c_float(softmax_scale), _ptr(out))
    if rc:
        raise ValueError(f"ref_seq_decode_attention rc={rc}")
    return out


# ---- sequences of different lengths in one batch: every batch element is a batch of one on its own slice of the planes

def _element(L: Layout, planes, b: int):
    return replace(L, batch=1), [p.reshape(L.batch, -1)[b] if p.size else p for p in planes]


def decode_attention_varlen(L: Layout, planes, q: np.ndarray, seq_lens, softmax_scale: float, bf16: bool = False) -> np.ndarray:
    """Batch element b attends over its first seq_lens[b] tokens (the uniform definition, element by element)."""
    q = np.ascontiguousarray(q)
    out = np.zeros((L.batch, q.shape[1], L.head_dim), dtype=np.float32)
    for b in range(L.batch):
        Lb, pb = _element(L, planes, b)
        out[b] = decode_attention(Lb, pb, q[b:b + 1], int(seq_lens[b]), softmax_scale, bf16)[0]
    return out


def quantize_append_at(L: Layout, planes, k_new: np.ndarray, v_new: np.ndarray, pos, bf16: bool = False) -> None:
    """One new token per batch element, stored at that element's own position pos[b]; k_new, v_new: [B, H, 1, D]."""
    for b in range(L.batch):
        Lb, pb = _element(L, planes, b)
        quantize_append(Lb, pb, np.ascontiguousarray(k_new[b:b + 1]), np.ascontiguousarray(v_new[b:b + 1]), int(pos[b]), bf16)


def seq_decode_attention_varlen(L: Layout, planes, q: np.ndarray, seq_lens, softmax_scale: float, bf16: bool = False) -> np.ndarray:
    """Channel-wise keys, one length per batch element: element b has had seq_lens[b] tokens appended and attends over
    all of them (its flushed blocks from the codes, the rest from its residual buffer)."""
    q = np.ascontiguousarray(q)
    out = np.zeros((L.batch, q.shape[1], L.head_dim), dtype=np.float32)
    for b in range(L.batch):
        Lb, pb = _element(L, planes, b)
        out[b] = seq_decode_attention(Lb, pb, q[b:b + 1], int(seq_lens[b]), softmax_scale, bf16)[0]
    return out


def seq_append_at(L: Layout, planes, k_new: np.ndarray, v_new: np.ndarray, pos, bf16: bool = False) -> None:
    """Channel-wise keys: one new token per batch element, element b having pos[b] tokens so far; k_new, v_new: [B, H, 1, D]."""
    for b in range(L.batch):
        Lb, pb = _element(L, planes, b)
        seq_append(Lb, pb, np.ascontiguousarray(k_new[b:b + 1]), np.ascontiguousarray(v_new[b:b + 1]), int(pos[b]), bf16)


# ---- paged planes: the same per-head layouts inside fixed-size pages of a pool, found through a page table

def paged_plane_bytes(L: Layout, page_tokens: int, n_pages: int):
    """Sizes of the four pool planes: n_pages pages, each holding page_tokens tokens of every KV head in the layout of a
    contiguous cache of that capacity."""
    one = plane_bytes(replace(L, batch=1, max_seq=page_tokens))
    return [n * n_pages for n in one]


def gather_pages(L: Layout, pool, table: np.ndarray, page_tokens: int, n_pages: int):
    """Contiguous planes (capacity = pages per sequence x page_tokens) assembled from the pool: logical page p of batch
    element b is pool page table[b][p]."""
    B, H = L.batch, L.kv_heads
    pages_per_seq = table.shape[1]
    out = []
    for plane in pool:
        if plane.size == 0:
            out.append(plane)
            continue
        per_head = plane.size // (n_pages * H)                 # bytes of one head's share of a page
        src = plane.reshape(n_pages, H, per_head)
        dst = np.zeros((B, H, pages_per_seq, per_head), dtype=np.uint8)
        for b in range(B):
            for p in range(pages_per_seq):
                dst[b, :, p] = src[table[b, p]]
        out.append(dst.reshape(-1))
    return out

"""CPU oracle (test infrastructure only) -- ctypes front end of ``alise_oracle.c``.

Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg of
``bench.py`` may import this package.  It shares nothing with the HIP path and
never imports it.

The C file states what is computed and cites the paper; this file only
marshals numpy arrays.  ``build()`` compiles the C file with gcc
(``-O2 -ffp-contract=off``: the compiler must not fuse or reorder the
quantizer's single-rounding fp32 steps).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "alise_oracle.c")
_LIB_PATH = os.path.join(_HERE, "libalise_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle into ``oracle/libalise_oracle.so``."""
    if (not force and os.path.exists(_LIB_PATH)
            and os.path.getmtime(_LIB_PATH) >= os.path.getmtime(_SRC)):
        return _LIB_PATH
    cmd = ["gcc", "-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
           "-shared", "-fPIC", "-o", _LIB_PATH, _SRC, "-lm"]
    subprocess.run(cmd, check=True)
    return _LIB_PATH


class _CCache(ctypes.Structure):
    _fields_ = [("k_codes", ctypes.c_void_p), ("v_codes", ctypes.c_void_p),
                ("k_meta", ctypes.c_void_p), ("v_meta", ctypes.c_void_p),
                ("num_pages", ctypes.c_int32), ("page_size", ctypes.c_int32),
                ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("bits", ctypes.c_int32), ("group_size", ctypes.c_int32)]


def lib():
    global _lib
    if _lib is None:
        build()
        L = ctypes.CDLL(_LIB_PATH)
        L.oracle_h2f.restype = ctypes.c_float
        L.oracle_h2f.argtypes = [ctypes.c_uint16]
        L.oracle_f2h_rne.restype = ctypes.c_uint16
        L.oracle_f2h_rne.argtypes = [ctypes.c_float]
        L.oracle_quant_group.restype = None
        L.oracle_quant_group.argtypes = [ctypes.c_void_p, ctypes.c_int, ctypes.c_int,
                                         ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.oracle_paged_prefill_attn.restype = ctypes.c_int
        L.oracle_paged_prefill_attn.argtypes = [ctypes.POINTER(_CCache), ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                                ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p, ctypes.c_int32,
                                                ctypes.c_int32, ctypes.c_double, ctypes.c_int32]
        L.oracle_kv_swap_bytes.restype = ctypes.c_size_t
        L.oracle_kv_swap_bytes.argtypes = [ctypes.POINTER(_CCache), ctypes.c_int32]
        L.oracle_kv_swap_out.restype = ctypes.c_int
        L.oracle_kv_swap_out.argtypes = [ctypes.POINTER(_CCache), ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p]
        L.oracle_kv_swap_in.restype = ctypes.c_int
        L.oracle_kv_swap_in.argtypes = [ctypes.POINTER(_CCache), ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p]
        L.oracle_kv_quant_write.restype = ctypes.c_int
        L.oracle_kv_quant_write.argtypes = [ctypes.POINTER(_CCache), ctypes.c_void_p, ctypes.c_void_p,
                                            ctypes.c_void_p, ctypes.c_int32]
        L.oracle_paged_decode_attn.restype = ctypes.c_int
        L.oracle_paged_decode_attn.argtypes = [ctypes.POINTER(_CCache), ctypes.c_void_p, ctypes.c_void_p,
                                               ctypes.c_void_p, ctypes.c_int32, ctypes.c_void_p,
                                               ctypes.c_int32, ctypes.c_int32, ctypes.c_double,
                                               ctypes.c_int32]
        L.oracle_kv_dequant_page.restype = ctypes.c_int
        L.oracle_kv_dequant_page.argtypes = [ctypes.POINTER(_CCache), ctypes.c_int32,
                                             ctypes.c_void_p, ctypes.c_void_p]
        L.oracle_d2h_rne.restype = ctypes.c_uint16
        L.oracle_d2h_rne.argtypes = [ctypes.c_double]
        L.oracle_add_layernorm.restype = ctypes.c_int
        L.oracle_add_layernorm.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_double,
                                           ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p, ctypes.c_void_p]
        L.oracle_bias_relu.restype = ctypes.c_int
        L.oracle_bias_relu.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int64, ctypes.c_int32, ctypes.c_void_p]
        L.oracle_dense_attn.restype = None
        L.oracle_dense_attn.argtypes = [ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
                                        ctypes.c_int, ctypes.c_int, ctypes.c_double, ctypes.c_void_p]
        _lib = L
    return _lib


def _ptr(a: np.ndarray) -> int:
    assert a.flags["C_CONTIGUOUS"]
    return a.ctypes.data


@dataclass
class Cache:
    """Host-side quantized paged cache in the canonical layout:
    codes uint8 [num_pages, Hkv, P, D*bits/8]; meta fp16 [num_pages, Hkv, P, D/G, 2]."""
    k_codes: np.ndarray
    v_codes: np.ndarray
    k_meta: np.ndarray
    v_meta: np.ndarray
    num_pages: int
    page_size: int
    num_kv_heads: int
    head_dim: int
    bits: int
    group_size: int

    @staticmethod
    def empty(num_pages, page_size, num_kv_heads, head_dim, bits, group_size, fill=0):
        cshape = (num_pages, num_kv_heads, page_size, head_dim * bits // 8)
        mshape = (num_pages, num_kv_heads, page_size, head_dim // group_size, 2)
        return Cache(np.full(cshape, fill, np.uint8), np.full(cshape, fill, np.uint8),
                     np.zeros(mshape, np.float16), np.zeros(mshape, np.float16),
                     num_pages, page_size, num_kv_heads, head_dim, bits, group_size)

    def _c(self) -> _CCache:
        return _CCache(_ptr(self.k_codes), _ptr(self.v_codes), _ptr(self.k_meta), _ptr(self.v_meta),
                       self.num_pages, self.page_size, self.num_kv_heads, self.head_dim,
                       self.bits, self.group_size)


def h2f(bits16: int) -> float:
    return float(lib().oracle_h2f(int(bits16)))


def f2h_rne(x: float) -> int:
    return int(lib().oracle_f2h_rne(ctypes.c_float(x)))


def quant_group(x: np.ndarray, bits: int):
    """x: fp16 [G] -> (codes uint8 [G], scale fp16 bits, zero fp16 bits)."""
    x = np.ascontiguousarray(x, dtype=np.float16)
    codes = np.zeros(x.size, np.uint8)
    sh = np.zeros(1, np.uint16)
    zh = np.zeros(1, np.uint16)
    lib().oracle_quant_group(_ptr(x), x.size, bits, _ptr(codes), _ptr(sh), _ptr(zh))
    return codes, int(sh[0]), int(zh[0])


def kv_quant_write(cache: Cache, k: np.ndarray, v: np.ndarray, slot_mapping: np.ndarray) -> None:
    k = np.ascontiguousarray(k, dtype=np.float16)
    v = np.ascontiguousarray(v, dtype=np.float16)
    slot_mapping = np.ascontiguousarray(slot_mapping, dtype=np.int64)
    T = slot_mapping.size
    assert k.shape == (T, cache.num_kv_heads, cache.head_dim) == v.shape
    cc = cache._c()
    rc = lib().oracle_kv_quant_write(ctypes.byref(cc), _ptr(k), _ptr(v), _ptr(slot_mapping), T)
    assert rc == 0


def paged_decode_attn(cache: Cache, q: np.ndarray, block_tables: np.ndarray,
                      context_lens: np.ndarray, softmax_scale: float, num_threads: int = 1) -> np.ndarray:
    """q fp16 [B, H, D] -> fp64 [B, H, D]."""
    q = np.ascontiguousarray(q, dtype=np.float16)
    block_tables = np.ascontiguousarray(block_tables, dtype=np.int32)
    context_lens = np.ascontiguousarray(context_lens, dtype=np.int32)
    B, H, D = q.shape
    assert D == cache.head_dim and H % cache.num_kv_heads == 0
    out = np.zeros((B, H, D), np.float64)
    cc = cache._c()
    rc = lib().oracle_paged_decode_attn(ctypes.byref(cc), _ptr(q), _ptr(out), _ptr(block_tables),
                                        block_tables.shape[1], _ptr(context_lens), B, H,
                                        float(softmax_scale), int(num_threads))
    assert rc == 0
    return out


def kv_dequant_page(cache: Cache, page: int):
    """-> fp16 (K, V), each [P, Hkv, D]."""
    shape = (cache.page_size, cache.num_kv_heads, cache.head_dim)
    k = np.zeros(shape, np.float16)
    v = np.zeros(shape, np.float16)
    cc = cache._c()
    rc = lib().oracle_kv_dequant_page(ctypes.byref(cc), int(page), _ptr(k), _ptr(v))
    assert rc == 0
    return k, v


def dense_attn(q: np.ndarray, K: np.ndarray, V: np.ndarray, softmax_scale: float) -> np.ndarray:
    """Unquantized attention for one head: q [D], K, V [L, D] (any float dtype) -> fp64 [D]."""
    q = np.ascontiguousarray(q, dtype=np.float64)
    K = np.ascontiguousarray(K, dtype=np.float64)
    V = np.ascontiguousarray(V, dtype=np.float64)
    L, D = K.shape
    out = np.zeros(D, np.float64)
    lib().oracle_dense_attn(_ptr(q), _ptr(K), _ptr(V), L, D, float(softmax_scale), _ptr(out))
    return out


def kv_swap_bytes(cache: Cache, num_tokens: int) -> int:
    c = cache._c()
    return int(lib().oracle_kv_swap_bytes(ctypes.byref(c), int(num_tokens)))


def kv_swap_out(cache: Cache, block_table: np.ndarray, num_tokens: int) -> np.ndarray:
    """Offloaded form (uint8 array) of the request whose pages ``block_table`` lists."""
    bt = np.ascontiguousarray(block_table, dtype=np.int32)
    c = cache._c()
    packed = np.zeros(kv_swap_bytes(cache, num_tokens), np.uint8)
    rc = lib().oracle_kv_swap_out(ctypes.byref(c), _ptr(bt), int(num_tokens), _ptr(packed))
    if rc:
        raise ValueError("block table entry out of range")
    return packed


def kv_swap_in(cache: Cache, block_table: np.ndarray, num_tokens: int, packed: np.ndarray) -> None:
    """Upload: write the offloaded form back into the pages ``block_table`` lists now."""
    bt = np.ascontiguousarray(block_table, dtype=np.int32)
    packed = np.ascontiguousarray(packed, dtype=np.uint8)
    assert packed.size >= kv_swap_bytes(cache, num_tokens)
    c = cache._c()
    rc = lib().oracle_kv_swap_in(ctypes.byref(c), _ptr(bt), int(num_tokens), _ptr(packed))
    if rc:
        raise ValueError("block table entry out of range")


def paged_prefill_attn(cache: Cache, q: np.ndarray, q_start: np.ndarray, block_tables: np.ndarray,
                       context_lens: np.ndarray, softmax_scale: float, num_threads: int = 0) -> np.ndarray:
    """q: fp16 [total_q, H, D], the requests' chunks back to back; q_start: int32 [B+1].
    Returns fp64 [total_q, H, D]: every query token attends causally over the cache."""
    q = np.ascontiguousarray(q, dtype=np.float16)
    qs = np.ascontiguousarray(q_start, dtype=np.int32)
    bt = np.ascontiguousarray(block_tables, dtype=np.int32)
    lens = np.ascontiguousarray(context_lens, dtype=np.int32)
    B = lens.shape[0]
    assert qs.shape == (B + 1,) and qs[0] == 0 and qs[-1] == q.shape[0]
    out = np.zeros(q.shape, np.float64)
    c = cache._c()
    if num_threads <= 0:
        num_threads = min(16, os.cpu_count() or 1)
    rc = lib().oracle_paged_prefill_attn(ctypes.byref(c), _ptr(q), _ptr(out), _ptr(qs), _ptr(bt), bt.shape[1],
                                         _ptr(lens), B, q.shape[1], float(softmax_scale), num_threads)
    if rc:
        raise ValueError("a chunk is longer than its request")
    return out


def d2h(x: float) -> int:
    """binary64 -> binary16 bit pattern, round to nearest even, one rounding."""
    return int(lib().oracle_d2h_rne(float(x)))


def add_layernorm(x, residual, gamma, beta, eps):
    """R19.  x, residual (or None): fp16 [rows, hidden]; gamma, beta: fp16 [hidden].
    Returns (h fp16 [rows, hidden], y fp64 [rows, hidden])."""
    x = np.ascontiguousarray(x, np.float16)
    rows, hidden = x.shape
    res = None if residual is None else np.ascontiguousarray(residual, np.float16)
    assert res is None or res.shape == x.shape
    gamma = np.ascontiguousarray(gamma, np.float16)
    beta = np.ascontiguousarray(beta, np.float16)
    assert gamma.shape == (hidden,) and beta.shape == (hidden,)
    h = np.empty((rows, hidden), np.float16)
    y = np.empty((rows, hidden), np.float64)
    rc = lib().oracle_add_layernorm(_ptr(x), None if res is None else _ptr(res), _ptr(gamma), _ptr(beta), float(eps),
                                    rows, hidden, _ptr(h), _ptr(y))
    if rc != 0:
        raise ValueError("oracle_add_layernorm: bad arguments")
    return h, y


def bias_relu(x, bias):
    """R20.  x: fp16 [rows, cols]; bias: fp16 [cols] or None.  Returns fp16 [rows, cols]."""
    x = np.ascontiguousarray(x, np.float16)
    rows, cols = x.shape
    b = None if bias is None else np.ascontiguousarray(bias, np.float16)
    assert b is None or b.shape == (cols,)
    y = np.empty((rows, cols), np.float16)
    rc = lib().oracle_bias_relu(_ptr(x), None if b is None else _ptr(b), rows, cols, _ptr(y))
    if rc != 0:
        raise ValueError("oracle_bias_relu: bad arguments")
    return y

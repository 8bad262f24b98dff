"""CPU oracle (test infrastructure only; see the header of ppd_oracle.c).

`build()` compiles ppd_oracle.c with gcc; `kv_append` / `mixed_attention` are ctypes wrappers over numpy
arrays of bf16 bit patterns (uint16).  `dense_attention` in bruteforce.py is a second, independent
implementation that never touches the page pool.
"""
import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ppd_oracle.c")
_LIB = os.path.join(_HERE, "libppd_oracle.so")
_lib = None


def build(force=False):
    """Compile the oracle (gcc -O2 -fopenmp; no fast-math, so the arithmetic is the source's)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(
            ["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


def _bind(path):
    """ctypes handle of an oracle build with the argument types set."""
    lib = ctypes.CDLL(path)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
    lib.ppd_oracle_kv_append.argtypes = [vp, vp, vp, vp, i64, i32, i32, i32, i64]
    lib.ppd_oracle_kv_append.restype = i32
    lib.ppd_oracle_mixed_attention.argtypes = [vp, vp, vp, i32, vp, vp, i32, i32, i32, i32, i32, i64,
                                               ctypes.c_float, vp, vp]
    lib.ppd_oracle_mixed_attention.restype = i32
    lib.ppd_oracle_kv_land.argtypes = [vp, vp, vp, i64, i32, vp, i64, i32, i32, i32, i64]
    lib.ppd_oracle_kv_land.restype = i32
    lib.ppd_oracle_transfer_delay.argtypes = [ctypes.c_double] * 4
    lib.ppd_oracle_transfer_delay.restype = ctypes.c_double
    f32 = ctypes.c_float
    lib.ppd_oracle_e4m3_value.argtypes = [ctypes.c_uint8]
    lib.ppd_oracle_e4m3_value.restype = ctypes.c_double
    lib.ppd_oracle_e4m3_code.argtypes = [f32]
    lib.ppd_oracle_e4m3_code.restype = ctypes.c_uint8
    lib.ppd_oracle_kv_append_fp8.argtypes = [vp, vp, vp, vp, i64, i32, i32, i32, i64, f32, f32]
    lib.ppd_oracle_kv_append_fp8.restype = i32
    lib.ppd_oracle_kv_land_fp8.argtypes = [vp, vp, vp, i64, i32, vp, i64, i32, i32, i32, i64, f32, f32]
    lib.ppd_oracle_kv_land_fp8.restype = i32
    lib.ppd_oracle_mixed_attention_fp8.argtypes = [vp, vp, f32, f32, vp, i32, vp, vp, i32, i32, i32, i32, i32, i64,
                                                   f32, vp, vp]
    lib.ppd_oracle_mixed_attention_fp8.restype = i32
    return lib


def _load():
    global _lib
    if _lib is None:
        build()
        _lib = _bind(_LIB)
    return _lib


def _ptr(a):
    return a.ctypes.data_as(ctypes.c_void_p)


def pool_elems(num_pages, Hkv, D, P):
    return int(num_pages) * 2 * Hkv * P * D


def kv_append(k, v, pool, slot_mapping, Hkv, D, P, num_pages):
    """In-place append of k, v ([T, Hkv, D] uint16) into pool (flat uint16) at slot_mapping ([T] int64)."""
    k = np.ascontiguousarray(k, dtype=np.uint16)
    v = np.ascontiguousarray(v, dtype=np.uint16)
    slot_mapping = np.ascontiguousarray(slot_mapping, dtype=np.int64)
    assert pool.dtype == np.uint16 and pool.flags.c_contiguous and pool.size == pool_elems(num_pages, Hkv, D, P)
    T = slot_mapping.shape[0]
    assert k.shape == (T, Hkv, D) and v.shape == (T, Hkv, D)
    rc = _load().ppd_oracle_kv_append(_ptr(k), _ptr(v), _ptr(pool), _ptr(slot_mapping), T, Hkv, D, P, num_pages)
    if rc != 0:
        raise ValueError("oracle kv_append: slot outside the pool")


def kv_land(k, v, pools, layer_stride, layers, slot_mapping, Hkv, D, P, num_pages):
    """In-place landing of k, v ([layers, T, Hkv, D] uint16) into `layers` pools laid out layer_stride apart."""
    k = np.ascontiguousarray(k, dtype=np.uint16)
    v = np.ascontiguousarray(v, dtype=np.uint16)
    slot_mapping = np.ascontiguousarray(slot_mapping, dtype=np.int64)
    T = slot_mapping.shape[0]
    assert k.shape == (layers, T, Hkv, D) and v.shape == k.shape
    assert pools.dtype == np.uint16 and pools.flags.c_contiguous
    assert layer_stride >= pool_elems(num_pages, Hkv, D, P) and pools.size >= layer_stride * (layers - 1) + pool_elems(
        num_pages, Hkv, D, P)
    rc = _load().ppd_oracle_kv_land(_ptr(k), _ptr(v), _ptr(pools), layer_stride, layers, _ptr(slot_mapping), T, Hkv, D,
                                    P, num_pages)
    if rc != 0:
        raise ValueError("oracle kv_land: slot outside the pool")


def transfer_delay(n_tokens, s_kv_bytes, beta_target, t_fast):
    return float(_load().ppd_oracle_transfer_delay(float(n_tokens), float(s_kv_bytes), float(beta_target), float(t_fast)))


def e4m3_value(code):
    """Value of an FP8 E4M3 code (0..255) as a Python float; NaN for the two NaN codes."""
    return float(_load().ppd_oracle_e4m3_value(int(code)))


def e4m3_code(y):
    """FP8 E4M3 code of a binary32 value: nearest, ties to the even code, saturating at 448."""
    return int(_load().ppd_oracle_e4m3_code(float(np.float32(y))))


def kv_append_fp8(k, v, pool, slot_mapping, Hkv, D, P, num_pages, k_scale, v_scale):
    """kv_append into FP8 pages: pool is flat uint8 of the same element count and layout."""
    k = np.ascontiguousarray(k, dtype=np.uint16)
    v = np.ascontiguousarray(v, dtype=np.uint16)
    slot_mapping = np.ascontiguousarray(slot_mapping, dtype=np.int64)
    assert pool.dtype == np.uint8 and pool.flags.c_contiguous and pool.size == pool_elems(num_pages, Hkv, D, P)
    T = slot_mapping.shape[0]
    assert k.shape == (T, Hkv, D) and v.shape == (T, Hkv, D)
    rc = _load().ppd_oracle_kv_append_fp8(_ptr(k), _ptr(v), _ptr(pool), _ptr(slot_mapping), T, Hkv, D, P, num_pages,
                                          float(k_scale), float(v_scale))
    if rc != 0:
        raise ValueError("oracle kv_append_fp8: slot outside the pool")


def kv_land_fp8(k, v, pools, layer_stride, layers, slot_mapping, Hkv, D, P, num_pages, k_scale, v_scale):
    """kv_land into FP8 pages (uint8 pools, layer_stride in elements)."""
    k = np.ascontiguousarray(k, dtype=np.uint16)
    v = np.ascontiguousarray(v, dtype=np.uint16)
    slot_mapping = np.ascontiguousarray(slot_mapping, dtype=np.int64)
    T = slot_mapping.shape[0]
    assert k.shape == (layers, T, Hkv, D) and v.shape == k.shape
    assert pools.dtype == np.uint8 and pools.flags.c_contiguous
    assert layer_stride >= pool_elems(num_pages, Hkv, D, P) and pools.size >= layer_stride * (layers - 1) + pool_elems(
        num_pages, Hkv, D, P)
    rc = _load().ppd_oracle_kv_land_fp8(_ptr(k), _ptr(v), _ptr(pools), layer_stride, layers, _ptr(slot_mapping), T, Hkv,
                                        D, P, num_pages, float(k_scale), float(v_scale))
    if rc != 0:
        raise ValueError("oracle kv_land_fp8: slot outside the pool")


def mixed_attention_fp8(q, pool, k_scale, v_scale, page_tables, L, n, Hq, Hkv, D, P, num_pages, scale, row_mask=None,
                        threads=None):
    """mixed_attention on FP8 pages (pool: flat uint8 codes)."""
    q = np.ascontiguousarray(q, dtype=np.uint16)
    page_tables = np.ascontiguousarray(page_tables, dtype=np.int32)
    L = np.ascontiguousarray(L, dtype=np.int32)
    n = np.ascontiguousarray(n, dtype=np.int32)
    B = L.shape[0]
    T = int(n.sum())
    assert q.shape == (T, Hq, D) and page_tables.shape[0] == B and n.shape[0] == B
    assert pool.dtype == np.uint8 and pool.flags.c_contiguous and pool.size == pool_elems(num_pages, Hkv, D, P)
    out = np.full((T, Hq, D), np.nan, dtype=np.float32)
    mask = None
    if row_mask is not None:
        mask = np.ascontiguousarray(row_mask, dtype=np.uint8)
        assert mask.shape == (T,)
    if threads is not None:
        os.environ["OMP_NUM_THREADS"] = str(int(threads))
    rc = _load().ppd_oracle_mixed_attention_fp8(
        _ptr(q), _ptr(pool), float(k_scale), float(v_scale), _ptr(page_tables),
        page_tables.shape[1] if page_tables.ndim == 2 else 0, _ptr(L), _ptr(n), B, Hq, Hkv, D, P, num_pages,
        float(scale), _ptr(mask) if mask is not None else None, _ptr(out))
    if rc != 0:
        raise ValueError("oracle mixed_attention_fp8: page table entry outside the pool (code %d)" % rc)
    return out


def mixed_attention(q, pool, page_tables, L, n, Hq, Hkv, D, P, num_pages, scale, row_mask=None, threads=None):
    """Returns out [T, Hq, D] float32.  q: [T, Hq, D] uint16 bf16 bits; rows masked out are left as NaN."""
    q = np.ascontiguousarray(q, dtype=np.uint16)
    page_tables = np.ascontiguousarray(page_tables, dtype=np.int32)
    L = np.ascontiguousarray(L, dtype=np.int32)
    n = np.ascontiguousarray(n, dtype=np.int32)
    B = L.shape[0]
    T = int(n.sum())
    assert q.shape == (T, Hq, D) and page_tables.shape[0] == B and n.shape[0] == B
    assert pool.dtype == np.uint16 and pool.flags.c_contiguous and pool.size == pool_elems(num_pages, Hkv, D, P)
    out = np.full((T, Hq, D), np.nan, dtype=np.float32)
    mask = None
    if row_mask is not None:
        mask = np.ascontiguousarray(row_mask, dtype=np.uint8)
        assert mask.shape == (T,)
    if threads is not None:
        os.environ["OMP_NUM_THREADS"] = str(int(threads))
    rc = _load().ppd_oracle_mixed_attention(
        _ptr(q), _ptr(pool), _ptr(page_tables), page_tables.shape[1] if page_tables.ndim == 2 else 0,
        _ptr(L), _ptr(n), B, Hq, Hkv, D, P, num_pages, float(scale),
        _ptr(mask) if mask is not None else None, _ptr(out))
    if rc != 0:
        raise ValueError("oracle mixed_attention: page table entry outside the pool (code %d)" % rc)
    return out

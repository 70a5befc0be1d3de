"""ctypes binding of the fp64 CPU oracle (oracle/hfx_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's CPU-baseline leg.  Nothing in the GPU library's package imports
this module, and this module imports nothing from that package.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hfx_oracle.c")
_LIB = os.path.join(_HERE, "libhfx_oracle.so")
_lib = None


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain C, OpenMP)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i32p = ctypes.POINTER(ctypes.c_int32)
        u16p = ctypes.POINTER(ctypes.c_uint16)
        f64p = ctypes.POINTER(ctypes.c_double)
        common = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_long, ctypes.c_double, ctypes.c_int,
                  i32p, i32p, i32p, i32p, i32p, u16p, u16p]
        lib.hfx_oracle_attention.argtypes = common + [f64p]
        lib.hfx_oracle_attention.restype = ctypes.c_int
        lib.hfx_oracle_attention_rows.argtypes = common + [ctypes.c_long, i32p, i32p, i32p, f64p]
        lib.hfx_oracle_attention_rows.restype = ctypes.c_int
        lib.hfx_oracle_gather_kv.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_long, ctypes.c_int,
                                             i32p, i32p, i32p, u16p, ctypes.c_int, u16p, u16p]
        lib.hfx_oracle_gather_kv.restype = ctypes.c_int
        lib.hfx_oracle_append_kv.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_long, ctypes.c_int, i32p, i32p,
                                             i32p, i32p, u16p, u16p, u16p]
        lib.hfx_oracle_append_kv.restype = ctypes.c_int
        lib.hfx_oracle_copy_pages.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_long, ctypes.c_long, ctypes.c_long,
                                              i32p, i32p, u16p, u16p]
        lib.hfx_oracle_copy_pages.restype = ctypes.c_int
        lib.hfx_oracle_num_threads.restype = ctypes.c_int
        _lib = lib
    return _lib


def _i32(a):
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32))


def _u16(a):
    a = np.ascontiguousarray(a, dtype=np.uint16)
    return a, a.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16))


def num_threads() -> int:
    return int(_load().hfx_oracle_num_threads())


def _common(Hq, Hkv, D, num_pages, scale, kind, q_len, ctx_len, bt_indptr, bt_pages, q, pool):
    keep = []
    args = [int(Hq), int(Hkv), int(D), int(num_pages), float(scale), int(len(kind))]
    for a in (kind, q_len, ctx_len, bt_indptr, bt_pages):
        arr, p = _i32(a)
        keep.append(arr)
        args.append(p)
    for a in (q, pool):
        arr, p = _u16(a)
        keep.append(arr)
        args.append(p)
    return args, keep


def attention(Hq, Hkv, D, num_pages, kind, q_len, ctx_len, bt_indptr, bt_pages, q, pool, scale=0.0):
    """Full step.  q, pool: uint16 bf16 bit patterns.  Returns float64 [T, Hq, D]."""
    args, keep = _common(Hq, Hkv, D, num_pages, scale, kind, q_len, ctx_len, bt_indptr, bt_pages, q, pool)
    T = int(np.asarray(q_len, dtype=np.int64).sum())
    out = np.zeros((T, Hq, D), dtype=np.float64)
    rc = _load().hfx_oracle_attention(*args, out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    if rc != 0:
        raise ValueError(f"oracle rejected the inputs (code {rc})")
    return out


def attention_rows(Hq, Hkv, D, num_pages, kind, q_len, ctx_len, bt_indptr, bt_pages, q, pool,
                   sample_req, sample_row, sample_head, scale=0.0):
    """Selected (request, chunk row, q-head) outputs.  Returns float64 [n, D]."""
    args, keep = _common(Hq, Hkv, D, num_pages, scale, kind, q_len, ctx_len, bt_indptr, bt_pages, q, pool)
    sr, psr = _i32(sample_req)
    sw, psw = _i32(sample_row)
    sh, psh = _i32(sample_head)
    out = np.zeros((len(sr), D), dtype=np.float64)
    rc = _load().hfx_oracle_attention_rows(*args, len(sr), psr, psw, psh,
                                           out.ctypes.data_as(ctypes.POINTER(ctypes.c_double)))
    if rc != 0:
        raise ValueError(f"oracle rejected the inputs (code {rc})")
    return out


def gather_kv(Hkv, D, num_pages, ctx_len, bt_indptr, bt_pages, pool, request):
    """Un-paged K, V of one request as uint16 [ctx_len, Hkv, D] (bit copies)."""
    cl, pcl = _i32(ctx_len)
    bi, pbi = _i32(bt_indptr)
    bp, pbp = _i32(bt_pages)
    pl, ppl = _u16(pool)
    c = int(cl[request])
    k = np.zeros((c, Hkv, D), dtype=np.uint16)
    v = np.zeros((c, Hkv, D), dtype=np.uint16)
    rc = _load().hfx_oracle_gather_kv(int(Hkv), int(D), int(num_pages), len(cl), pcl, pbi, pbp, ppl,
                                      int(request), k.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)),
                                      v.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)))
    if rc != 0:
        raise ValueError(f"oracle rejected the inputs (code {rc})")
    return k, v


def attention_batch(b, scale=0.0):
    """Convenience: any object with the step's fields (num_q_heads, ..., q, pool)."""
    return attention(b.num_q_heads, b.num_kv_heads, b.head_dim, b.num_pages, b.kind, b.q_len, b.ctx_len,
                     b.bt_indptr, b.bt_pages, b.q, b.pool, scale)


def attention_rows_batch(b, sample_req, sample_row, sample_head, scale=0.0):
    return attention_rows(b.num_q_heads, b.num_kv_heads, b.head_dim, b.num_pages, b.kind, b.q_len, b.ctx_len,
                          b.bt_indptr, b.bt_pages, b.q, b.pool, sample_req, sample_row, sample_head, scale)


def append_kv(Hkv, D, num_pages, q_len, ctx_len, bt_indptr, bt_pages, k_new, v_new, pool):
    """Writes the chunk tokens' K/V (uint16 [T, Hkv, D]) into `pool` in place (pool must be a contiguous
    uint16 array)."""
    ql, pql = _i32(q_len)
    cl, pcl = _i32(ctx_len)
    bi, pbi = _i32(bt_indptr)
    bp, pbp = _i32(bt_pages)
    kn, pkn = _u16(k_new)
    vn, pvn = _u16(v_new)
    assert pool.dtype == np.uint16 and pool.flags.c_contiguous
    rc = _load().hfx_oracle_append_kv(int(Hkv), int(D), int(num_pages), len(ql), pql, pcl, pbi, pbp, pkn, pvn,
                                      pool.ctypes.data_as(ctypes.POINTER(ctypes.c_uint16)))
    if rc != 0:
        raise ValueError(f"oracle rejected the inputs (code {rc})")


def copy_pages(Hkv, D, src_ids, dst_ids, src_pool, dst_pool):
    """dst_pool[dst_ids[i]] = src_pool[src_ids[i]] (whole pages, in place on dst_pool; both contiguous uint16
    arrays whose leading axis is the page)."""
    si, psi = _i32(src_ids)
    di, pdi = _i32(dst_ids)
    assert len(si) == len(di)
    assert src_pool.dtype == np.uint16 and src_pool.flags.c_contiguous
    assert dst_pool.dtype == np.uint16 and dst_pool.flags.c_contiguous
    u16p = ctypes.POINTER(ctypes.c_uint16)
    rc = _load().hfx_oracle_copy_pages(int(Hkv), int(D), src_pool.shape[0], dst_pool.shape[0], len(si), psi, pdi,
                                       src_pool.ctypes.data_as(u16p), dst_pool.ctypes.data_as(u16p))
    if rc != 0:
        raise ValueError(f"oracle rejected the inputs (code {rc})")

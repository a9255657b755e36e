"""fp64 CPU oracle for prefix-reuse prefill -- TEST INFRASTRUCTURE.

Thin ctypes front end of ``pbkv_oracle.c`` (the arithmetic lives there).  Only
the tests, the smoke check and the benchmark's ``cpu_baseline`` leg may import
this package; the GPU library never does and shares no code with it.

Arrays are numpy: ``float32`` for the fp32 configuration, ``uint16`` holding
bf16 bit patterns for the bf16 ones.
"""
import ctypes
import os

import numpy as np

from . import build as _build

_LIB = None


def _bind(path):
    if not path:
        raise ImportError("the oracle library is not built (oracle/build.py)")
    lib = ctypes.CDLL(path)
    vp, i32, i64 = ctypes.c_void_p, ctypes.c_int, ctypes.c_int64
    lib.pbkv_oracle_prefill.restype = ctypes.c_int
    lib.pbkv_oracle_prefill.argtypes = [i32, i32, i32, i32, i32, i32, i64, i32,
                                        vp, vp, vp, vp, vp, vp, vp, vp, i64, vp, vp, vp]
    lib.pbkv_oracle_append.restype = ctypes.c_int
    lib.pbkv_oracle_append.argtypes = [i32, i32, i32, i32, i32, i64, i32,
                                       vp, vp, vp, vp, vp, vp]
    lib.pbkv_oracle_swap_in.restype = ctypes.c_int
    lib.pbkv_oracle_swap_in.argtypes = [i64, i64, vp, vp, i64, vp]
    lib.pbkv_oracle_swap_out.restype = ctypes.c_int
    lib.pbkv_oracle_swap_out.argtypes = [i64, i64, vp, vp, i64, vp]
    lib.pbkv_oracle_threads.restype = ctypes.c_int
    lib.pbkv_oracle_set_threads.restype = None
    lib.pbkv_oracle_set_threads.argtypes = [ctypes.c_int]
    return lib


def threads():
    """Host threads the oracle's row loop uses."""
    return int(_lib().pbkv_oracle_threads())


def set_threads(n):
    """Host threads the row loop uses from now on (results do not depend on it)."""
    _lib().pbkv_oracle_set_threads(int(n))


def _lib():
    global _LIB
    if _LIB is None:
        _LIB = _bind(_build.build(force=False))
    return _LIB


def _dtype_code(a):
    if a.dtype == np.uint16:
        return 0
    if a.dtype == np.float32:
        return 1
    raise TypeError("oracle takes uint16 (bf16 bits) or float32 arrays, got %s" % a.dtype)


def _c(a, dtype=None):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a, a.ctypes.data_as(ctypes.c_void_p)


def prefill(q, k_new, v_new, kv_pool, block_table, prefix_lens, new_lens, rows=None,
            want_stats=False):
    """softmax(q K^T / sqrt(d)) V of each suffix row over prefix pages + own suffix.

    q [N,Hq,d]; k_new, v_new [N,Hkv,d]; kv_pool [num_pages,2,Hkv,P,d];
    block_table [B,max_pages] int32; prefix_lens, new_lens [B] int32.
    ``rows``: optional packed row indices to evaluate (all rows if None).
    Returns out float64 [n_out,Hq,d] (and rowsum, lse [n_out,Hq] if want_stats).
    """
    code = _dtype_code(q)
    for a in (k_new, v_new, kv_pool):
        if _dtype_code(a) != code:
            raise TypeError("mixed dtypes")
    N, Hq, d = q.shape
    num_pages, two, Hkv, P, d2 = kv_pool.shape
    assert two == 2 and d2 == d and k_new.shape == (N, Hkv, d) and v_new.shape == (N, Hkv, d)
    B, max_pages = block_table.shape
    q, qp = _c(q)
    k_new, kp = _c(k_new)
    v_new, vp = _c(v_new)
    kv_pool, pp = _c(kv_pool)
    block_table, bp = _c(block_table, np.int32)
    prefix_lens, plp = _c(prefix_lens, np.int32)
    new_lens, nlp = _c(new_lens, np.int32)
    assert prefix_lens.shape == (B,) and new_lens.shape == (B,)
    assert int(new_lens.sum()) == N
    if rows is None:
        n_out, rp = N, None
    else:
        rows, rp = _c(rows, np.int64)
        n_out = rows.shape[0]
    out = np.empty((n_out, Hq, d), np.float64)
    rowsum = np.empty((n_out, Hq), np.float64)
    lse = np.empty((n_out, Hq), np.float64)
    rc = _lib().pbkv_oracle_prefill(code, B, Hq, Hkv, d, P, num_pages, max_pages,
                                    qp, kp, vp, pp, bp, plp, nlp, rp, n_out,
                                    out.ctypes.data_as(ctypes.c_void_p),
                                    rowsum.ctypes.data_as(ctypes.c_void_p),
                                    lse.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError("oracle rejected its arguments (code %d)" % rc)
    return (out, rowsum, lse) if want_stats else out


def append_kv(k_new, v_new, kv_pool, block_table, prefix_lens, new_lens):
    """Return a copy of ``kv_pool`` with the suffix K/V scattered to their pages."""
    N, Hkv, d = k_new.shape
    num_pages, two, Hkv2, P, d2 = kv_pool.shape
    assert two == 2 and Hkv2 == Hkv and d2 == d and v_new.shape == k_new.shape
    assert k_new.dtype == v_new.dtype == kv_pool.dtype
    B, max_pages = block_table.shape
    pool = np.array(kv_pool, copy=True, order="C")
    k_new, kp = _c(k_new)
    v_new, vp = _c(v_new)
    block_table, bp = _c(block_table, np.int32)
    prefix_lens, plp = _c(prefix_lens, np.int32)
    new_lens, nlp = _c(new_lens, np.int32)
    assert int(new_lens.sum()) == N
    rc = _lib().pbkv_oracle_append(pool.dtype.itemsize, B, Hkv, d, P, num_pages, max_pages,
                                   kp, vp, pool.ctypes.data_as(ctypes.c_void_p), bp, plp, nlp)
    if rc != 0:
        raise ValueError("oracle rejected its arguments (code %d)" % rc)
    return pool


def swap_in(host_pages, page_ids, kv_pool):
    """Return a copy of ``kv_pool`` with host page i written to pool page page_ids[i]."""
    pool = np.array(kv_pool, copy=True, order="C")
    num_pages = pool.shape[0]
    page_bytes = pool[0].nbytes if num_pages else 0
    host_pages, hp = _c(host_pages)
    page_ids, ip = _c(page_ids, np.int32)
    n = page_ids.shape[0]
    assert host_pages.dtype == pool.dtype and host_pages.size * host_pages.itemsize == n * page_bytes
    rc = _lib().pbkv_oracle_swap_in(page_bytes, num_pages, hp, ip, n,
                                    pool.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError("oracle rejected its arguments (code %d)" % rc)
    return pool


def swap_out(kv_pool, page_ids):
    """Return host pages [n][...page shape]: host page i is a copy of pool page page_ids[i]."""
    pool, pp = _c(kv_pool)
    num_pages = pool.shape[0]
    page_bytes = pool[0].nbytes if num_pages else 0
    page_ids, ip = _c(page_ids, np.int32)
    n = page_ids.shape[0]
    host = np.zeros((n,) + pool.shape[1:], pool.dtype)
    rc = _lib().pbkv_oracle_swap_out(page_bytes, num_pages, pp, ip, n,
                                     host.ctypes.data_as(ctypes.c_void_p))
    if rc != 0:
        raise ValueError("oracle rejected its arguments (code %d)" % rc)
    return host


def decode(q, kv_pool, block_table, context_lens):
    """Paged decode attention (Sec. 4.3: the pure-decode steps behind which prefetch transfers
    are hidden): one query row per request attends to the request's first context_lens[r]
    cached tokens, all read through the block table.  This is the prefill definition above
    with one new token whose own K/V are the pool's entries at position L-1; requests with
    context_lens[r] == 0 give a zero row.  q: [B, Hq, d]; returns float64 [B, Hq, d]."""
    pool = np.asarray(kv_pool)
    lens = np.asarray(context_lens, np.int64)
    B, P = lens.shape[0], pool.shape[3]
    Hkv, d = pool.shape[2], pool.shape[4]
    live = np.nonzero(lens > 0)[0]
    out = np.zeros((B,) + tuple(np.asarray(q).shape[1:]), np.float64)
    if live.size == 0:
        return out
    k_last = np.zeros((live.size, Hkv, d), pool.dtype)
    v_last = np.zeros((live.size, Hkv, d), pool.dtype)
    for i, r in enumerate(live):
        pos = int(lens[r]) - 1
        pg = int(np.asarray(block_table)[r, pos // P])
        k_last[i] = pool[pg, 0, :, pos % P]
        v_last[i] = pool[pg, 1, :, pos % P]
    res = prefill(np.asarray(q)[live], k_last, v_last, pool, np.asarray(block_table)[live],
                  (lens[live] - 1).astype(np.int32), np.ones(live.size, np.int32))
    out[live] = res
    return out

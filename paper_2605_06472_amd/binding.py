"""ctypes binding of libpbkv.so: same names as the C boundary, argument marshalling only.

Every operation runs in the HIP kernels of the library.  There is no CPU or PyTorch
fallback: if the library has not been built, or a call fails, an exception is raised.
Tensors may be torch tensors (anything with ``data_ptr()``) or raw integer addresses;
``prefix_lens`` / ``new_lens`` / ``page_ids`` are host int32 arrays.
"""
import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libpbkv.so")

PBKV_BF16, PBKV_F32 = 0, 1
STATUS = {0: "PBKV_OK", -1: "PBKV_ERR_NULL", -2: "PBKV_ERR_SHAPE", -3: "PBKV_ERR_DTYPE",
          -4: "PBKV_ERR_RANGE", -5: "PBKV_ERR_ALIAS", -6: "PBKV_ERR_DEVICE", -7: "PBKV_ERR_LIMIT"}


class PbkvError(RuntimeError):
    def __init__(self, code, message):
        super().__init__("%s (%d): %s" % (STATUS.get(code, "?"), code, message))
        self.code = code


class Shape(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("num_q_heads", ctypes.c_int32),
                ("num_kv_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("page_size", ctypes.c_int32), ("num_pages", ctypes.c_int32),
                ("max_pages_per_req", ctypes.c_int32), ("dtype", ctypes.c_int32)]


_lib = None


def load():
    """Load libpbkv.so (built by paper_2605_06472_amd.build); raises if it is missing."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise ImportError("libpbkv.so is not built: run `python -m paper_2605_06472_amd.build` "
                              "(there is no fallback path)")
        lib = ctypes.CDLL(LIB_PATH)
        vp, i32p = ctypes.c_void_p, ctypes.c_void_p
        sp = ctypes.POINTER(Shape)
        lib.pbkv_prefix_prefill.restype = ctypes.c_int
        lib.pbkv_prefix_prefill.argtypes = [sp, vp, vp, vp, vp, i32p, i32p, i32p, vp, vp]
        lib.pbkv_append_kv.restype = ctypes.c_int
        lib.pbkv_append_kv.argtypes = [sp, vp, vp, vp, i32p, i32p, i32p, vp]
        lib.pbkv_swap_in_pages.restype = ctypes.c_int
        lib.pbkv_swap_in_pages.argtypes = [sp, vp, i32p, ctypes.c_int32, vp, vp]
        lib.pbkv_paged_decode.restype = ctypes.c_int
        lib.pbkv_paged_decode.argtypes = [sp, vp, vp, i32p, i32p, vp, vp]
        lib.pbkv_paged_decode_static.restype = ctypes.c_int
        lib.pbkv_paged_decode_static.argtypes = [sp, vp, vp, i32p, i32p, vp, vp]
        lib.pbkv_swap_out_pages.restype = ctypes.c_int
        lib.pbkv_swap_out_pages.argtypes = [sp, vp, i32p, ctypes.c_int32, vp, vp]
        lib.pbkv_gather_probe.restype = ctypes.c_int
        lib.pbkv_gather_probe.argtypes = [sp, vp, vp, vp, i32p, i32p, i32p, vp, ctypes.c_int64,
                                          ctypes.POINTER(ctypes.c_int64), ctypes.POINTER(ctypes.c_int32), vp]
        lib.pbkv_set_attn_waves.restype = ctypes.c_int
        lib.pbkv_set_attn_waves.argtypes = [ctypes.c_int]
        lib.pbkv_page_bytes.restype = ctypes.c_int64
        lib.pbkv_page_bytes.argtypes = [sp]
        lib.pbkv_last_error.restype = ctypes.c_char_p
        lib.pbkv_version.restype = ctypes.c_char_p
        _lib = lib
    return _lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return ctypes.c_void_p(t)
    return ctypes.c_void_p(t.data_ptr())


def _host_i32(a):
    if hasattr(a, "data_ptr") and not isinstance(a, np.ndarray):      # torch CPU tensor
        a = a.numpy()
    a = np.ascontiguousarray(a, dtype=np.int32)
    return a, ctypes.c_void_p(a.ctypes.data)


def _stream(stream):
    if stream is None:
        import torch
        return ctypes.c_void_p(torch.cuda.current_stream().cuda_stream)
    if isinstance(stream, int):
        return ctypes.c_void_p(stream)
    return ctypes.c_void_p(stream.cuda_stream)


def _check(rc):
    if rc != 0:
        raise PbkvError(rc, load().pbkv_last_error().decode())


def make_shape(batch, num_q_heads, num_kv_heads, head_dim, page_size, num_pages,
               max_pages_per_req, dtype):
    code = {"bf16": PBKV_BF16, "f32": PBKV_F32}.get(dtype, dtype)
    return Shape(batch, num_q_heads, num_kv_heads, head_dim, page_size, num_pages,
                 max_pages_per_req, code)


def page_bytes(shape):
    return int(load().pbkv_page_bytes(ctypes.byref(shape)))


def version():
    return load().pbkv_version().decode()


def set_attn_waves(waves):
    """4, 8 or 64: work-group shape of every later bf16 attention launch; 0: the library chooses."""
    _check(load().pbkv_set_attn_waves(int(waves)))


def prefix_prefill(shape, q, k_new, v_new, kv_pool, block_table, prefix_lens, new_lens, out,
                   stream=None):
    pl, plp = _host_i32(prefix_lens)
    nl, nlp = _host_i32(new_lens)
    _check(load().pbkv_prefix_prefill(ctypes.byref(shape), _ptr(q), _ptr(k_new), _ptr(v_new),
                                      _ptr(kv_pool), _ptr(block_table), plp, nlp, _ptr(out),
                                      _stream(stream)))


def append_kv(shape, k_new, v_new, kv_pool, block_table, prefix_lens, new_lens, stream=None):
    pl, plp = _host_i32(prefix_lens)
    nl, nlp = _host_i32(new_lens)
    _check(load().pbkv_append_kv(ctypes.byref(shape), _ptr(k_new), _ptr(v_new), _ptr(kv_pool),
                                 _ptr(block_table), plp, nlp, _stream(stream)))


def swap_in_pages(shape, host_pages, page_ids, kv_pool, stream=None):
    ids, idp = _host_i32(page_ids)
    _check(load().pbkv_swap_in_pages(ctypes.byref(shape), _ptr(host_pages), idp,
                                     int(ids.shape[0]), _ptr(kv_pool), _stream(stream)))


def paged_decode(shape, q, kv_pool, block_table, context_lens, out, stream=None):
    cl, clp = _host_i32(context_lens)
    _check(load().pbkv_paged_decode(ctypes.byref(shape), _ptr(q), _ptr(kv_pool), _ptr(block_table), clp,
                                    _ptr(out), _stream(stream)))


def paged_decode_static(shape, q, kv_pool, block_table, context_lens, out, stream=None):
    cl, clp = _host_i32(context_lens)
    _check(load().pbkv_paged_decode_static(ctypes.byref(shape), _ptr(q), _ptr(kv_pool), _ptr(block_table), clp,
                                           _ptr(out), _stream(stream)))


def swap_out_pages(shape, kv_pool, page_ids, host_pages, stream=None):
    ids, idp = _host_i32(page_ids)
    _check(load().pbkv_swap_out_pages(ctypes.byref(shape), _ptr(kv_pool), idp, int(ids.shape[0]),
                                      _ptr(host_pages), _stream(stream)))


def gather_probe(shape, k_new, v_new, kv_pool, block_table, prefix_lens, new_lens, unit_xor=None,
                 stream=None):
    """Returns (n_units, unit_tokens).  ``unit_xor`` is a device 32-bit integer tensor that
    receives one word per unit; None only asks for the two numbers."""
    pl, plp = _host_i32(prefix_lens)
    nl, nlp = _host_i32(new_lens)
    n_units, unit_tokens = ctypes.c_int64(0), ctypes.c_int32(0)
    cap = 0 if unit_xor is None else int(unit_xor.numel())
    _check(load().pbkv_gather_probe(ctypes.byref(shape), _ptr(k_new), _ptr(v_new), _ptr(kv_pool),
                                    _ptr(block_table), plp, nlp, _ptr(unit_xor), cap,
                                    ctypes.byref(n_units), ctypes.byref(unit_tokens),
                                    None if unit_xor is None else _stream(stream)))
    return n_units.value, unit_tokens.value

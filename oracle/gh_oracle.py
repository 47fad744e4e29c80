"""ctypes front end of oracle/gh_oracle.c.

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg, never by the product package.  It imports numpy
and the standard library, nothing from the HIP side.

All 16-bit tensors travel as numpy uint16 arrays holding the raw bit patterns
(dtype code 0 = IEEE binary16, 1 = bfloat16); results come back as float64.
Every function cites the passage of the paper its C counterpart follows in
gh_oracle.c's header: Section 2.1 (stage F2), Appendix A Table 5 (per-head
Q.K then A.V), Section 4.3 (FP32-or-better arithmetic, MHA with GQA), Section
4.1.3 (slot id and latest-token position), footnote of Section 2.2 (split
along the sequence and merge).
"""
import ctypes as C
import os

import numpy as np

from .build import LIB, build_oracle

F16, BF16 = 0, 1


class Problem(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("dtype", C.c_int32), ("n_slots", C.c_int32),
        ("slot_capacity", C.c_int32),
        ("slot_stride", C.c_int64), ("head_stride", C.c_int64), ("row_stride", C.c_int64),
        ("scale", C.c_double),
        ("block_rows", C.c_int32), ("block_stride", C.c_int64),
    ]


_lib = None


def lib():
    global _lib
    if _lib is None:
        if not os.path.exists(LIB):
            build_oracle()
        L = C.CDLL(LIB)
        L.gho_f16_to_f64.restype = C.c_double
        L.gho_f16_to_f64.argtypes = [C.c_uint16]
        L.gho_bf16_to_f64.restype = C.c_double
        L.gho_bf16_to_f64.argtypes = [C.c_uint16]
        L.gho_num_threads.restype = C.c_int
        L.gho_set_num_threads.argtypes = [C.c_int]
        _lib = L
    return _lib


def _u16(a):
    a = np.ascontiguousarray(a)
    assert a.dtype == np.uint16, a.dtype
    return a


def _i32(a):
    return np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def _ptr(a):
    return a.ctypes.data_as(C.c_void_p)


def make_problem(batch, n_q_heads, n_kv_heads, head_dim, dtype, n_slots, slot_capacity,
                 scale, strides=None, block=(0, 0)):
    """Cache layout defaults to [slot][kv head][row][d]; strides are in elements; `block` =
    (rows per block, elements between a head's blocks) for blocked layouts."""
    if strides is None:
        strides = (n_kv_heads * slot_capacity * head_dim, slot_capacity * head_dim, head_dim)
    assert n_q_heads % n_kv_heads == 0
    return Problem(batch, n_q_heads, n_kv_heads, head_dim, dtype, n_slots, slot_capacity,
                   strides[0], strides[1], strides[2], float(scale), int(block[0]), int(block[1]))


def num_threads():
    return lib().gho_num_threads()


def set_num_threads(n):
    lib().gho_set_num_threads(int(n))


def widen(bits, dtype):
    """Exact float64 value of each 16-bit pattern (element-wise, slow path through C)."""
    bits = np.asarray(bits, dtype=np.uint16)
    f = lib().gho_bf16_to_f64 if dtype == BF16 else lib().gho_f16_to_f64
    return np.array([f(int(x)) for x in bits.ravel()], dtype=np.float64).reshape(bits.shape)


def kv_append(p, k_cache, v_cache, k_new, v_new, slot_id, pos):
    """In-place append into the host mirror; returns the number of skipped sequences."""
    assert k_cache.dtype == np.uint16 and v_cache.dtype == np.uint16
    assert k_cache.flags.c_contiguous and v_cache.flags.c_contiguous
    k_new, v_new, slot_id, pos = _u16(k_new), _u16(v_new), _i32(slot_id), _i32(pos)
    skipped = C.c_int32(0)
    lib().gho_kv_append(C.byref(p), _ptr(k_cache), _ptr(v_cache), _ptr(k_new), _ptr(v_new),
                        _ptr(slot_id), _ptr(pos), C.byref(skipped))
    return skipped.value


def decode_attention(p, q, k_cache, v_cache, slot_id, ctx_len):
    """softmax(scale * q K^T) V per (sequence, head) in float64 -> [B, H, d]."""
    q, k_cache, v_cache = _u16(q), _u16(k_cache), _u16(v_cache)
    slot_id, ctx_len = _i32(slot_id), _i32(ctx_len)
    out = np.empty((p.batch, p.n_q_heads, p.head_dim), dtype=np.float64)
    lib().gho_decode_attention(C.byref(p), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                               _ptr(slot_id), _ptr(ctx_len), _ptr(out))
    return out


def partial(p, q, k_cache, v_cache, slot_id, b, h, r0, r1):
    """(m, l, o[d]) of rows [r0, r1) in the base-2 form used by the merge."""
    q, k_cache, v_cache, slot_id = _u16(q), _u16(k_cache), _u16(v_cache), _i32(slot_id)
    m, l = C.c_double(0), C.c_double(0)
    o = np.empty(p.head_dim, dtype=np.float64)
    lib().gho_partial(C.byref(p), _ptr(q), _ptr(k_cache), _ptr(v_cache), _ptr(slot_id),
                      C.c_int32(b), C.c_int32(h), C.c_int32(r0), C.c_int32(r1),
                      C.byref(m), C.byref(l), _ptr(o))
    return m.value, l.value, o


def merge(m, l, o):
    """Merge n partial results: m[n], l[n], o[n, d] -> out[d]."""
    m = np.ascontiguousarray(m, dtype=np.float64)
    l = np.ascontiguousarray(l, dtype=np.float64)
    o = np.ascontiguousarray(o, dtype=np.float64)
    n, d = o.shape
    out = np.empty(d, dtype=np.float64)
    lib().gho_merge(C.c_int32(n), C.c_int32(d), _ptr(m), _ptr(l), _ptr(o), _ptr(out))
    return out

"""Thin ctypes binding of libgh_tier2.so (argument marshalling only).

Function names and argument order are those of include/gh_tier2.h.  Tensors
are torch device tensors whose data pointers are handed to the library; the
stream is torch's current HIP stream unless one is given.  There is no CPU
path: if the library has not been built this module raises on first use.
"""
import ctypes as C
import os

import torch

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libgh_tier2.so")

GH_OK = 0
GH_ERR_NULL, GH_ERR_SHAPE, GH_ERR_UNSUPPORTED = -1, -2, -3
GH_ERR_WORKSPACE, GH_ERR_CAPACITY, GH_ERR_HIP = -4, -5, -6
GH_F16, GH_BF16 = 0, 1
GH_KERNEL_AUTO, GH_KERNEL_VALU, GH_KERNEL_MFMA = 0, 1, 2
GH_DEV_BAD_SLOT, GH_DEV_BAD_POS = 1, 2

EXPORTS = ("gh_status_string", "gh_decode_chunk_rows", "gh_decode_num_chunks",
           "gh_decode_workspace_bytes", "gh_kv_append", "gh_decode_attention", "gh_decode_reduce")


class gh_problem(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("dtype", C.c_int32), ("n_slots", C.c_int32),
        ("slot_capacity", C.c_int32), ("max_ctx_len", C.c_int32),
        ("slot_stride", C.c_int64), ("head_stride", C.c_int64), ("row_stride", C.c_int64),
        ("scale", C.c_float), ("chunk_rows", C.c_int32), ("kernel", C.c_int32),
    ]


class GhError(RuntimeError):
    def __init__(self, status):
        self.status = status
        super().__init__(f"gh_tier2: status {status}: {gh_status_string(status)}")


_lib = None


def lib():
    """Load the HIP library; a missing build is an error, never a fallback."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it first (python -c 'import __graft_entry__ as g; g.build()')")
        L = C.CDLL(LIB_PATH)
        P = C.POINTER(gh_problem)
        V = C.c_void_p
        L.gh_status_string.restype = C.c_char_p
        L.gh_status_string.argtypes = [C.c_int32]
        L.gh_decode_chunk_rows.restype = C.c_int32
        L.gh_decode_chunk_rows.argtypes = [P]
        L.gh_decode_num_chunks.restype = C.c_int32
        L.gh_decode_num_chunks.argtypes = [P]
        L.gh_decode_workspace_bytes.restype = C.c_size_t
        L.gh_decode_workspace_bytes.argtypes = [P]
        L.gh_kv_append.restype = C.c_int32
        L.gh_kv_append.argtypes = [P, V, V, V, V, V, V, V, V]
        L.gh_decode_attention.restype = C.c_int32
        L.gh_decode_attention.argtypes = [P, V, V, V, V, V, V, C.c_size_t, V]
        L.gh_decode_reduce.restype = C.c_int32
        L.gh_decode_reduce.argtypes = [P, V, V, V, V]
        _lib = L
    return _lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return t
    return t.data_ptr()


def _stream(stream):
    if stream is None:
        return torch.cuda.current_stream().cuda_stream
    if isinstance(stream, int):
        return stream
    return stream.cuda_stream


def make_problem(batch, n_q_heads, n_kv_heads, head_dim, dtype, n_slots, slot_capacity,
                 max_ctx_len, strides, scale, chunk_rows=0, kernel=GH_KERNEL_AUTO):
    return gh_problem(batch, n_q_heads, n_kv_heads, head_dim, dtype, n_slots, slot_capacity,
                      max_ctx_len, strides[0], strides[1], strides[2], scale, chunk_rows, kernel)


def gh_status_string(status):
    return lib().gh_status_string(int(status)).decode()


def gh_decode_chunk_rows(p):
    return lib().gh_decode_chunk_rows(C.byref(p))


def gh_decode_num_chunks(p):
    return lib().gh_decode_num_chunks(C.byref(p))


def gh_decode_workspace_bytes(p):
    return lib().gh_decode_workspace_bytes(C.byref(p))


def gh_kv_append(p, k_cache, v_cache, k_new, v_new, slot_id, pos, dev_status=None, stream=None):
    return lib().gh_kv_append(C.byref(p), _ptr(k_cache), _ptr(v_cache), _ptr(k_new), _ptr(v_new),
                              _ptr(slot_id), _ptr(pos), _ptr(dev_status), _stream(stream))


def gh_decode_attention(p, q, k_cache, v_cache, slot_id, ctx_len, workspace, workspace_bytes=None,
                        stream=None):
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    return lib().gh_decode_attention(C.byref(p), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                     _ptr(slot_id), _ptr(ctx_len), _ptr(workspace),
                                     workspace_bytes, _stream(stream))


def gh_decode_reduce(p, workspace, ctx_len, out, stream=None):
    return lib().gh_decode_reduce(C.byref(p), _ptr(workspace), _ptr(ctx_len), _ptr(out),
                                  _stream(stream))


def check(status):
    if status != GH_OK:
        raise GhError(status)


def problem_from_inputs(inp, chunk_rows=0, kernel=GH_KERNEL_AUTO, max_ctx_len=None):
    """gh_problem for a dict made by workloads.make_inputs."""
    w = inp["workload"]
    dtype = GH_BF16 if w.dtype == "bf16" else GH_F16
    if max_ctx_len is None:
        max_ctx_len = int(inp["lengths"].max()) + 1
    return make_problem(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, dtype, inp["n_slots"],
                        inp["capacity"], max_ctx_len, inp["strides"], inp["scale"], chunk_rows,
                        kernel)


def alloc_workspace(p, device="cuda"):
    """A float32 device tensor of gh_decode_workspace_bytes(p) bytes (at least one element)."""
    n = gh_decode_workspace_bytes(p)
    return torch.empty(max(n // 4, 1), dtype=torch.float32, device=device)


def decode_step(p, inp, workspace, out, dev_status=None, stream=None, append=True):
    """append -> attention -> reduce on one stream; raises on a host-side error."""
    if append:
        check(gh_kv_append(p, inp["k_cache"], inp["v_cache"], inp["k_new"], inp["v_new"],
                           inp["slot_id"], inp["pos"], dev_status, stream))
    check(gh_decode_attention(p, inp["q"], inp["k_cache"], inp["v_cache"], inp["slot_id"],
                              inp["ctx_len"], workspace, None, stream))
    check(gh_decode_reduce(p, workspace, inp["ctx_len"], out, stream))
    return out

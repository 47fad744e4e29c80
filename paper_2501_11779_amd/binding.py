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
GH_ERR_WORKSPACE, GH_ERR_CAPACITY, GH_ERR_HIP, GH_ERR_SCRATCH = -4, -5, -6, -7
GH_STATIC_SCRATCH_BYTES = 64 << 20
GH_F16, GH_BF16 = 0, 1
GH_KERNEL_AUTO, GH_KERNEL_VALU, GH_KERNEL_MFMA, GH_KERNEL_STRIPS = 0, 1, 2, 3
GH_DEV_BAD_SLOT, GH_DEV_BAD_POS = 1, 2

EXPORTS = ("gh_status_string", "gh_decode_chunk_rows", "gh_decode_num_chunks",
           "gh_decode_workspace_bytes", "gh_kv_append", "gh_decode_attention", "gh_decode_reduce",
           "gh_decode_reduce_native", "gh_decode_split_plan", "gh_decode_attention_out",
           "gh_decode_attention_static", "gh_decode_step", "gh_decode_step_init")
GH_OUT_F32, GH_OUT_NATIVE = 0, 1
GH_PROBE_STORE_PLAIN, GH_PROBE_STORE_NT, GH_PROBE_STORE_WRITE_THROUGH = 0, 1, 2
POOL_EXPORTS = ("gh_slot_pool_create", "gh_slot_pool_create_host_only", "gh_slot_pool_destroy", "gh_slot_pool_k", "gh_slot_pool_v",
                "gh_slot_pool_strides", "gh_slot_pool_reserve", "gh_slot_pool_release",
                "gh_slot_pool_mapped_rows", "gh_slot_pool_get_stats", "gh_slot_pool_blocks")
GH_POOL_TOKEN_MAJOR, GH_POOL_HEAD_BLOCKED = 0, 1
POOL_LAYOUTS = {"token_major": GH_POOL_TOKEN_MAJOR, "head_blocked": GH_POOL_HEAD_BLOCKED}


class gh_problem(C.Structure):
    _fields_ = [
        ("batch", C.c_int32), ("n_q_heads", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("dtype", C.c_int32), ("n_slots", C.c_int32),
        ("slot_capacity", C.c_int32), ("max_ctx_len", C.c_int32),
        ("slot_stride", C.c_int64), ("head_stride", C.c_int64), ("row_stride", C.c_int64),
        ("scale", C.c_float), ("chunk_rows", C.c_int32), ("kernel", C.c_int32),
        ("q_batch_stride", C.c_int64), ("new_batch_stride", C.c_int64),
        ("block_rows", C.c_int32), ("tokens_per_group", C.c_int32), ("block_stride", C.c_int64),
    ]


class gh_split_plan(C.Structure):
    _fields_ = [("balanced", C.c_int32), ("n_workers", C.c_int32), ("min_share", C.c_int32),
                ("passes_per_strip", C.c_int32), ("strips_per_kv_head", C.c_int32),
                ("n_chunks", C.c_int32), ("waves_per_worker", C.c_int32),
                ("groups_per_launch", C.c_int32)]


class gh_slot_pool_config(C.Structure):
    _fields_ = [
        ("n_slots", C.c_int32), ("slot_capacity", C.c_int32), ("n_kv_heads", C.c_int32),
        ("head_dim", C.c_int32), ("page_rows", C.c_int32), ("device", C.c_int32),
        ("layout", C.c_int32), ("physical_pages", C.c_int64),
    ]


class gh_slot_pool_stats(C.Structure):
    _fields_ = [
        ("page_bytes", C.c_int64), ("virtual_bytes", C.c_int64), ("physical_bytes", C.c_int64),
        ("pages_total", C.c_int64), ("pages_mapped", C.c_int64),
        ("slot_capacity", C.c_int32), ("slots_in_use", C.c_int32), ("pages_created", C.c_int64),
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
        L.gh_decode_split_plan.restype = C.c_int32
        L.gh_decode_split_plan.argtypes = [P, C.POINTER(gh_split_plan)]
        L.gh_decode_workspace_bytes.restype = C.c_size_t
        L.gh_decode_workspace_bytes.argtypes = [P]
        L.gh_kv_append.restype = C.c_int32
        L.gh_kv_append.argtypes = [P, V, V, V, V, V, V, V, V]
        L.gh_decode_attention.restype = C.c_int32
        L.gh_decode_attention.argtypes = [P, V, V, V, V, V, V, C.c_size_t, V]
        L.gh_decode_attention_out.restype = C.c_int32
        L.gh_decode_attention_out.argtypes = [P, V, V, V, V, V, V, C.c_size_t, V, C.c_int32, V]
        L.gh_decode_attention_static.restype = C.c_int32
        L.gh_decode_attention_static.argtypes = [P, V, V, V, V, V, V, C.c_int32, V]
        L.gh_decode_step_init.restype = C.c_int32
        L.gh_decode_step_init.argtypes = [P, V, C.c_size_t, V]
        L.gh_decode_step.restype = C.c_int32
        L.gh_decode_step.argtypes = [P, V, V, V, V, V, V, V, V, C.c_size_t, V, C.c_int32, V, V]
        L.gh_decode_reduce.restype = C.c_int32
        L.gh_decode_reduce.argtypes = [P, V, V, V, V]
        L.gh_decode_reduce_native.restype = C.c_int32
        L.gh_decode_reduce_native.argtypes = [P, V, V, V, V]
        L.gh_probe_stream_read.restype = C.c_int32
        L.gh_probe_stream_read.argtypes = [V, C.c_size_t, C.c_int32, C.c_int32, C.c_int32, V, V, V]
        I32P = C.POINTER(C.c_int32)
        I64P = C.POINTER(C.c_int64)
        L.gh_slot_pool_create.restype = C.c_int32
        L.gh_slot_pool_create.argtypes = [C.POINTER(gh_slot_pool_config), C.POINTER(V)]
        L.gh_slot_pool_create_host_only.restype = C.c_int32
        L.gh_slot_pool_create_host_only.argtypes = [C.POINTER(gh_slot_pool_config), C.c_int64, C.POINTER(V)]
        L.gh_slot_pool_destroy.restype = C.c_int32
        L.gh_slot_pool_destroy.argtypes = [V]
        L.gh_slot_pool_k.restype = V
        L.gh_slot_pool_k.argtypes = [V]
        L.gh_slot_pool_v.restype = V
        L.gh_slot_pool_v.argtypes = [V]
        L.gh_slot_pool_blocks.restype = C.c_int32
        L.gh_slot_pool_blocks.argtypes = [V, C.POINTER(C.c_int32), I64P]
        L.gh_slot_pool_strides.restype = C.c_int32
        L.gh_slot_pool_strides.argtypes = [V, I64P, I64P, I64P]
        L.gh_slot_pool_reserve.restype = C.c_int32
        L.gh_slot_pool_reserve.argtypes = [V, I32P, I32P, C.c_int32]
        L.gh_slot_pool_release.restype = C.c_int32
        L.gh_slot_pool_release.argtypes = [V, I32P, C.c_int32]
        L.gh_slot_pool_mapped_rows.restype = C.c_int32
        L.gh_slot_pool_mapped_rows.argtypes = [V, C.c_int32]
        L.gh_slot_pool_get_stats.restype = C.c_int32
        L.gh_slot_pool_get_stats.argtypes = [V, C.POINTER(gh_slot_pool_stats)]
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
                 max_ctx_len, strides, scale, chunk_rows=0, kernel=GH_KERNEL_AUTO,
                 q_batch_stride=0, new_batch_stride=0, block=(0, 0), tokens_per_group=0):
    return gh_problem(batch, n_q_heads, n_kv_heads, head_dim, dtype, n_slots, slot_capacity,
                      max_ctx_len, strides[0], strides[1], strides[2], scale, chunk_rows, kernel,
                      q_batch_stride, new_batch_stride, int(block[0]), int(tokens_per_group),
                      int(block[1]))


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


def gh_decode_attention_out(p, q, k_cache, v_cache, slot_id, ctx_len, workspace, out, out_kind,
                            workspace_bytes=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    return lib().gh_decode_attention_out(C.byref(p), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                         _ptr(slot_id), _ptr(ctx_len), _ptr(workspace),
                                         workspace_bytes, _ptr(out), int(out_kind), _stream(stream))


def gh_decode_attention_static(p, q, k_cache, v_cache, slot_id, ctx_len, out, out_kind, stream=None):
    return lib().gh_decode_attention_static(C.byref(p), _ptr(q), _ptr(k_cache), _ptr(v_cache),
                                            _ptr(slot_id), _ptr(ctx_len), _ptr(out), int(out_kind),
                                            _stream(stream))


def gh_decode_step_init(p, workspace, workspace_bytes=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    return lib().gh_decode_step_init(C.byref(p), _ptr(workspace), workspace_bytes, _stream(stream))


def gh_decode_step(p, q, k_new, v_new, k_cache, v_cache, slot_id, pos, workspace, out, out_kind,
                   dev_status=None, workspace_bytes=None, stream=None):
    if workspace_bytes is None:
        workspace_bytes = workspace.numel() * workspace.element_size()
    return lib().gh_decode_step(C.byref(p), _ptr(q), _ptr(k_new), _ptr(v_new), _ptr(k_cache),
                                _ptr(v_cache), _ptr(slot_id), _ptr(pos), _ptr(workspace),
                                workspace_bytes, _ptr(out), int(out_kind), _ptr(dev_status),
                                _stream(stream))


def gh_decode_reduce(p, workspace, ctx_len, out, stream=None):
    return lib().gh_decode_reduce(C.byref(p), _ptr(workspace), _ptr(ctx_len), _ptr(out),
                                  _stream(stream))


def gh_decode_reduce_native(p, workspace, ctx_len, out16, stream=None):
    return lib().gh_decode_reduce_native(C.byref(p), _ptr(workspace), _ptr(ctx_len), _ptr(out16),
                                         _stream(stream))


def gh_decode_split_plan(p):
    out = gh_split_plan()
    check(lib().gh_decode_split_plan(C.byref(p), C.byref(out)))
    return out


def gh_probe_stream_read(src, nbytes, n_waves, store_every, store_policy, rec, sink, stream=None):
    """Measurement aid of include/gh_probe.h (stream = 0 is accepted without a GPU for the host-side
    argument checks)."""
    return lib().gh_probe_stream_read(_ptr(src), int(nbytes), int(n_waves), int(store_every),
                                      int(store_policy), _ptr(rec), _ptr(sink),
                                      0 if stream == 0 else _stream(stream))


def check(status):
    if status != GH_OK:
        raise GhError(status)


def problem_from_inputs(inp, chunk_rows=0, kernel=GH_KERNEL_AUTO, max_ctx_len=None,
                        tokens_per_group=0):
    """gh_problem for a dict made by workloads.make_inputs."""
    w = inp["workload"]
    dtype = GH_BF16 if w.dtype == "bf16" else GH_F16
    if max_ctx_len is None:
        max_ctx_len = int(inp["lengths"].max()) + 1
    return make_problem(w.batch, w.n_q_heads, w.n_kv_heads, w.head_dim, dtype, inp["n_slots"],
                        inp["capacity"], max_ctx_len, inp["strides"], inp["scale"], chunk_rows,
                        kernel, block=inp.get("block", (0, 0)), tokens_per_group=tokens_per_group)


def alloc_workspace(p, device="cuda"):
    """A float32 device tensor of gh_decode_workspace_bytes(p) bytes (at least one element)."""
    n = gh_decode_workspace_bytes(p)
    return torch.empty(max(n // 4, 1), dtype=torch.float32, device=device)


def decode_step(p, inp, workspace, out, dev_status=None, stream=None, append=True, early=False):
    """append -> attention -> reduce on one stream; raises on a host-side error.  `out` is fp32 or
    the problem's 16-bit type; `early` lets the attention kernel store the heads it can finish."""
    native = out.dtype != torch.float32
    if append:
        check(gh_kv_append(p, inp["k_cache"], inp["v_cache"], inp["k_new"], inp["v_new"],
                           inp["slot_id"], inp["pos"], dev_status, stream))
    if early:
        check(gh_decode_attention_out(p, inp["q"], inp["k_cache"], inp["v_cache"], inp["slot_id"],
                                      inp["ctx_len"], workspace, out,
                                      GH_OUT_NATIVE if native else GH_OUT_F32, None, stream))
    else:
        check(gh_decode_attention(p, inp["q"], inp["k_cache"], inp["v_cache"], inp["slot_id"],
                                  inp["ctx_len"], workspace, None, stream))
    check((gh_decode_reduce_native if native else gh_decode_reduce)(p, workspace, inp["ctx_len"],
                                                                    out, stream))
    return out


def alloc_step_workspace(p, device="cuda", stream=None):
    """A workspace for gh_decode_step: allocated and its arrival counters cleared."""
    ws = alloc_workspace(p, device)
    check(gh_decode_step_init(p, ws, None, stream))
    return ws


def decode_step_one_launch(p, inp, workspace, out, dev_status=None, stream=None):
    """gh_decode_step on a make_inputs() dict; `workspace` from alloc_step_workspace()."""
    check(gh_decode_step(p, inp["q"], inp["k_new"], inp["v_new"], inp["k_cache"], inp["v_cache"],
                         inp["slot_id"], inp["pos"], workspace, out,
                         GH_OUT_F32 if out.dtype == torch.float32 else GH_OUT_NATIVE, dev_status,
                         None, stream))
    return out


# ----------------------------------------------------------------------------- paged context slots
def _i32_array(values):
    arr = (C.c_int32 * len(values))(*[int(v) for v in values])
    return arr, len(values)


class _DeviceArrayView:
    """Lets torch wrap a raw device address (no copy, no ownership)."""

    def __init__(self, ptr, shape):
        self.__cuda_array_interface__ = {"shape": tuple(shape), "typestr": "<i2", "data": (ptr, False),
                                         "version": 2}


class SlotPool:
    """Marshalling front end of gh_slot_pool_* (include/gh_slot_pool.h)."""

    def __init__(self, n_slots, slot_capacity, n_kv_heads, head_dim, page_rows, physical_pages,
                 device=0, layout="token_major", host_only_fail_at=None):
        self._h = C.c_void_p()
        cfg = gh_slot_pool_config(n_slots, slot_capacity, n_kv_heads, head_dim, page_rows, device,
                                  POOL_LAYOUTS[layout], physical_pages)
        self.layout = layout
        if host_only_fail_at is None:
            check(lib().gh_slot_pool_create(C.byref(cfg), C.byref(self._h)))
        else:       # bookkeeping only, no GPU (gh_slot_pool_create_host_only)
            check(lib().gh_slot_pool_create_host_only(C.byref(cfg), int(host_only_fail_at),
                                                      C.byref(self._h)))
        self.n_slots, self.n_kv_heads, self.head_dim = n_slots, n_kv_heads, head_dim
        self.page_rows = page_rows
        self.capacity = self.stats().slot_capacity

    def close(self):
        if self._h:
            h, self._h = self._h, C.c_void_p()
            check(lib().gh_slot_pool_destroy(h))

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    @property
    def k_ptr(self):
        return lib().gh_slot_pool_k(self._h)

    @property
    def v_ptr(self):
        return lib().gh_slot_pool_v(self._h)

    @property
    def strides(self):
        a, b, c = C.c_int64(), C.c_int64(), C.c_int64()
        check(lib().gh_slot_pool_strides(self._h, C.byref(a), C.byref(b), C.byref(c)))
        return (a.value, b.value, c.value)

    @property
    def block(self):
        """(block_rows, block_stride) for gh_problem."""
        r, s = C.c_int32(), C.c_int64()
        check(lib().gh_slot_pool_blocks(self._h, C.byref(r), C.byref(s)))
        return (r.value, s.value)

    def reserve(self, slot_ids, rows):
        s, n = _i32_array(slot_ids)
        r, _ = _i32_array(rows)
        return lib().gh_slot_pool_reserve(self._h, s, r, n)

    def release(self, slot_ids):
        s, n = _i32_array(slot_ids)
        return lib().gh_slot_pool_release(self._h, s, n)

    def mapped_rows(self, slot):
        return lib().gh_slot_pool_mapped_rows(self._h, int(slot))

    def stats(self):
        st = gh_slot_pool_stats()
        check(lib().gh_slot_pool_get_stats(self._h, C.byref(st)))
        return st

    def rows_view(self, which, slot, rows, dtype):
        """Torch view [rows, H_kv, d] of the first `rows` rows of a slot; they must be reserved.
        In the head-blocked layout `rows` counts whole pages and the view is a permutation of the
        pages' [page][H_kv][page_rows][d] storage (not contiguous, but writable in place)."""
        assert 0 <= rows <= self.mapped_rows(slot)
        base = self.k_ptr if which == "k" else self.v_ptr
        ptr = base + slot * self.strides[0] * 2
        if self.layout == "head_blocked":
            assert rows % self.page_rows == 0
            shape = (rows // self.page_rows, self.n_kv_heads, self.page_rows, self.head_dim)
            view = torch.as_tensor(_DeviceArrayView(ptr, shape), device="cuda").view(dtype)
            return view.permute(0, 2, 1, 3)          # [page][row in page][H_kv][d]
        view = torch.as_tensor(_DeviceArrayView(ptr, (rows, self.n_kv_heads, self.head_dim)),
                               device="cuda")
        return view.view(dtype)

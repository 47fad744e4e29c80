"""gh_decode_attention_static: the entry point for callers that cannot allocate.

Its partial records live in a buffer inside the library's code object, so it takes no workspace.
It must give the bits of gh_decode_attention_out + merge (the same kernels on a caller's
workspace), stay within the benchmark spec's tolerance of the oracle, and survive being called again
with a smaller problem while the buffer still holds the larger call's records.
"""
import ctypes as C

import numpy as np
import pytest
import torch

from paper_2501_11779_amd import binding as G
from paper_2501_11779_amd import workloads as W
from tests import helpers as Hh

DEV = "cuda"


def _with_workspace(p, inp, dt, append):
    w = inp["workload"]
    ws = G.alloc_workspace(p, DEV)
    ws.fill_(float("nan"))
    out = torch.full((w.batch, w.n_q_heads, 128), float("nan"), dtype=dt, device=DEV)
    G.decode_step(p, inp, ws, out, append=append, early=True)
    torch.cuda.synchronize()
    return out


def _static(p, inp, dt):
    w = inp["workload"]
    out = torch.full((w.batch, w.n_q_heads, 128), float("nan"), dtype=dt, device=DEV)
    G.check(G.gh_decode_attention_static(p, inp["q"], inp["k_cache"], inp["v_cache"], inp["slot_id"],
                                         inp["ctx_len"], out,
                                         G.GH_OUT_F32 if dt == torch.float32 else G.GH_OUT_NATIVE))
    torch.cuda.synchronize()
    return out


@pytest.mark.gpu
@pytest.mark.parametrize("native", [False, True])
def test_static_scratch_call_matches_the_workspace_call_twice_in_a_row(native):
    big = W.Workload("static_big", 96, 32, 4, 128, "bf16", ("uniform", 0, 900), 501)
    small = W.Workload("static_small", 5, 32, 4, 128, "bf16", ("uniform", 0, 200), 502)
    for w in (big, small):                        # the second call finds the first one's records
        inp = W.make_inputs(w, DEV)
        host = Hh.host_copy(inp)
        p = G.problem_from_inputs(inp)
        assert G.gh_decode_workspace_bytes(p) <= G.GH_STATIC_SCRATCH_BYTES
        dt = W.TORCH_DTYPE[w.dtype] if native else torch.float32
        print(f"{w.name}: B={w.batch} workspace={G.gh_decode_workspace_bytes(p)} B native={native}",
              flush=True)
        want = _with_workspace(p, inp, dt, append=True)
        got = _static(p, inp, dt)
        view = torch.int16 if native else torch.int32
        assert torch.equal(got.cpu().view(view), want.cpu().view(view))
        if not native:
            Hh.assert_parity(got.cpu().numpy(), Hh.oracle_step(inp, host), w.name)


@pytest.mark.gpu
def test_static_scratch_call_on_a_fixed_split_and_the_vector_kernel():
    w = W.Workload("static_fixed", 9, 8, 2, 128, "f16", ("uniform", 0, 500), 503)
    inp = W.make_inputs(w, DEV)
    host = Hh.host_copy(inp)
    want = None
    for kernel, chunk_rows in ((G.GH_KERNEL_MFMA, 128), (G.GH_KERNEL_VALU, 0)):
        p = G.problem_from_inputs(inp, chunk_rows=chunk_rows, kernel=kernel)
        ref = _with_workspace(p, inp, torch.float32, append=want is None)
        got = _static(p, inp, torch.float32)
        assert torch.equal(got.cpu().view(torch.int32), ref.cpu().view(torch.int32))
        if want is None:
            want = Hh.oracle_step(inp, host)
        Hh.assert_parity(got.cpu().numpy(), want, f"static kernel={kernel}")


def test_problem_beyond_the_static_scratch_is_refused_before_anything_runs():
    """Host-side check only: no GPU call happens before the size is judged."""
    p = G.make_problem(1024, 64, 8, 128, G.GH_BF16, 1024, 4097, 4097,
                       (8 * 4097 * 128, 4097 * 128, 128), 128 ** -0.5)
    assert G.gh_decode_workspace_bytes(p) > G.GH_STATIC_SCRATCH_BYTES
    fake = 1 << 20                                 # non-null, 16-byte aligned, never dereferenced
    st = G.lib().gh_decode_attention_static(C.byref(p), fake, fake, fake, fake, fake, fake,
                                            G.GH_OUT_F32, None)
    assert st == G.GH_ERR_SCRATCH
    assert "static scratch" in G.gh_status_string(st)
    assert G.lib().gh_decode_attention_static(C.byref(p), fake, fake, fake, fake, fake, None,
                                              G.GH_OUT_F32, None) == G.GH_ERR_NULL
    assert G.lib().gh_decode_attention_static(C.byref(p), fake, fake, fake, fake, fake, fake, 5,
                                              None) == G.GH_ERR_UNSUPPORTED

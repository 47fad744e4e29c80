"""Paged context slots (HIP virtual memory): bookkeeping, oversubscription, parity on the GPU."""
import numpy as np
import pytest
import torch

from paper_2501_11779_amd import binding as G
from paper_2501_11779_amd import workloads as W
from paper_2501_11779_amd.paged import into_pool, pages_needed
from tests import helpers as Hh

pytestmark = pytest.mark.gpu
DEV = "cuda"


def test_pool_bookkeeping_and_oversubscription():
    pool = G.SlotPool(n_slots=8, slot_capacity=1000, n_kv_heads=2, head_dim=128, page_rows=256,
                      physical_pages=10)
    st = pool.stats()
    assert st.slot_capacity == 1024 and pool.capacity == 1024
    assert st.page_bytes == 256 * 2 * 128 * 2
    assert st.virtual_bytes == 2 * 8 * 1024 * 2 * 128 * 2
    assert st.physical_bytes == 2 * 10 * st.page_bytes
    assert st.virtual_bytes / st.physical_bytes == pytest.approx(3.2)      # oversubscribed
    assert st.pages_mapped == 0 and st.slots_in_use == 0
    assert pool.strides == (1024 * 256, 128, 256)

    assert pool.reserve([3, 0, 5, 7], [300, 1, 1024, 0]) == G.GH_OK       # 2 + 1 + 4 + 0 pages
    assert [pool.mapped_rows(s) for s in (3, 0, 5, 7, 1)] == [512, 256, 1024, 0, 0]
    assert pool.stats().pages_mapped == 7 and pool.stats().slots_in_use == 3
    assert pool.reserve([3], [200]) == G.GH_OK                            # already covered
    assert pool.stats().pages_mapped == 7

    # all or nothing: 3 free pages cannot cover 4 more
    assert pool.reserve([1, 2], [512, 512]) == G.GH_ERR_CAPACITY
    assert pool.stats().pages_mapped == 7 and pool.mapped_rows(1) == 0
    assert pool.reserve([1], [1025]) == G.GH_ERR_CAPACITY                  # beyond a slot
    assert pool.reserve([8], [1]) == G.GH_ERR_SHAPE
    assert pool.reserve([1], [768]) == G.GH_OK                             # exactly the rest
    assert pool.stats().pages_mapped == 10
    assert pool.reserve([2], [1]) == G.GH_ERR_CAPACITY

    assert pool.release([5]) == G.GH_OK                                    # pages go back
    assert pool.mapped_rows(5) == 0 and pool.stats().pages_mapped == 6
    assert pool.reserve([2], [1024]) == G.GH_OK
    assert pool.stats().pages_mapped == 10
    assert pool.release([0, 1, 2, 3, 5, 7]) == G.GH_OK
    assert pool.stats().pages_mapped == 0 and pool.stats().slots_in_use == 0
    pool.close()


def test_create_leaves_the_current_device_alone_and_creates_pages_on_demand():
    import ctypes
    hip = ctypes.CDLL("libamdhip64.so")
    dev = ctypes.c_int(-1)
    assert hip.hipGetDevice(ctypes.byref(dev)) == 0
    before = dev.value
    pool = G.SlotPool(n_slots=4, slot_capacity=1000, n_kv_heads=2, head_dim=128, page_rows=256,
                      physical_pages=1000)                   # a budget far beyond what is used
    assert hip.hipGetDevice(ctypes.byref(dev)) == 0 and dev.value == before
    assert torch.cuda.current_device() == before
    st = pool.stats()
    assert st.pages_created == 0 and st.pages_total == 1000
    assert pool.reserve([1], [300]) == G.GH_OK
    assert pool.stats().pages_created == 2 and pool.stats().pages_mapped == 2
    assert pool.release([1]) == G.GH_OK
    assert pool.reserve([2], [100]) == G.GH_OK               # reuses a page that exists
    assert pool.stats().pages_created == 2
    pool.close()


def test_pool_refuses_bad_configurations():
    with pytest.raises(G.GhError) as e:
        G.SlotPool(0, 100, 2, 128, 256, 4)
    assert e.value.status == G.GH_ERR_SHAPE
    with pytest.raises(G.GhError) as e:
        G.SlotPool(4, 100, 2, 64, 256, 4)
    assert e.value.status == G.GH_ERR_UNSUPPORTED
    with pytest.raises(G.GhError) as e:          # 3 rows * 1 head * 256 B is not a whole granule
        G.SlotPool(4, 100, 1, 128, 3, 4)
    assert e.value.status == G.GH_ERR_UNSUPPORTED


def _first_rows(pool, which, slot, n, dt):
    """Bits of rows [0, n) of a slot as [n, H_kv, d], whatever the pool's layout."""
    view = pool.rows_view(which, slot, pool.mapped_rows(slot), dt)
    return W.bits(view.reshape(-1, pool.n_kv_heads, pool.head_dim)[:n])


def test_head_blocked_pool_reports_its_geometry():
    pool = G.SlotPool(4, 1000, 2, 128, 256, physical_pages=4, layout="head_blocked")
    assert pool.capacity == 1024
    assert pool.strides == (1024 * 256, 256 * 128, 128)
    assert pool.block == (256, 256 * 2 * 128)
    pool.close()
    pool = G.SlotPool(4, 1000, 2, 128, 256, physical_pages=4)
    assert pool.block == (0, 0)
    pool.close()


@pytest.mark.parametrize("layout", ["token_major", "head_blocked"])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_decode_step_on_paged_slots_matches_oracle(dtype, layout):
    lengths = np.array([0, 255, 256, 257, 700, 31, 1023], dtype=np.int32)
    w = W.Workload("paged", len(lengths), 8, 2, 128, dtype, ("const", 0), 71)
    inp = W.make_inputs(w, DEV, lengths=lengths, n_slots=12, capacity=1024, layout="token_major")
    host = Hh.host_copy(inp)
    need = pages_needed(lengths, 256)
    pool = G.SlotPool(12, 1024, 2, 128, 256, physical_pages=need, layout=layout)   # none to spare
    assert pool.stats().virtual_bytes / pool.stats().physical_bytes > 3.0
    paged = into_pool(pool, inp)
    assert pool.stats().pages_mapped == need

    p = G.problem_from_inputs(paged)
    ws = G.alloc_workspace(p, DEV)
    ws.fill_(float("nan"))
    out = torch.full((w.batch, 8, 128), float("nan"), dtype=torch.float32, device=DEV)
    G.decode_step(p, paged, ws, out)
    torch.cuda.synchronize()
    want = Hh.oracle_step(inp, host)                                       # same layout, host mirror
    Hh.assert_parity(out.cpu().numpy(), want, "paged")
    # the appended rows, and everything before them, are the oracle's mirror bit for bit
    dt = W.TORCH_DTYPE[dtype]
    for b in range(w.batch):
        s, n = int(inp["slots"][b]), int(lengths[b]) + 1
        assert np.array_equal(_first_rows(pool, "k", s, n, dt), host["k_cache"][s, :n])
        assert np.array_equal(_first_rows(pool, "v", s, n, dt), host["v_cache"][s, :n])
    pool.close()


@pytest.mark.parametrize("layout", ["token_major", "head_blocked"])
def test_slots_grow_page_by_page_and_are_reused(layout):
    """Decode steps push a sequence across a page border; a finished prompt's slot is taken over."""
    w = W.Workload("grow", 2, 4, 2, 128, "bf16", ("const", 0), 72)
    lengths = np.array([254, 40], dtype=np.int32)
    inp = W.make_inputs(w, DEV, lengths=lengths, n_slots=3, capacity=512, layout="token_major")
    host = Hh.host_copy(inp)
    pool = G.SlotPool(3, 512, 2, 128, 256, physical_pages=3, layout=layout)
    paged = into_pool(pool, inp)
    assert pool.stats().pages_mapped == 2
    out = torch.empty((2, 4, 128), dtype=torch.float32, device=DEV)
    for step in range(4):                        # rows 254..257 of sequence 0: crosses row 256
        pos = lengths + step
        assert pool.reserve(inp["slots"], pos + 1) == G.GH_OK
        paged["pos"] = torch.from_numpy(pos.copy()).to(DEV)
        paged["ctx_len"] = (paged["pos"] + 1).to(torch.int32)
        host["pos"], host["ctx_len"] = pos.copy(), pos + 1
        p = G.problem_from_inputs(paged, max_ctx_len=int(pos.max()) + 1)
        ws = G.alloc_workspace(p, DEV)
        G.decode_step(p, paged, ws, out)
        torch.cuda.synchronize()
        Hh.assert_parity(out.cpu().numpy(), Hh.oracle_step(inp, host), f"step {step}")
    assert pool.stats().pages_mapped == 3 and pool.mapped_rows(int(inp["slots"][0])) == 512
    # prompt 1 finishes: its slot is reused from position 0 without a release, as in the paper
    assert pool.reserve([int(inp["slots"][1])], [1]) == G.GH_OK
    assert pool.stats().pages_mapped == 3
    pool.close()

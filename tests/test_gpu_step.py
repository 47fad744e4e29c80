"""gh_decode_step: append + attention + merge in one launch, against the oracle.

The appended rows must land bit for bit, the result must meet the benchmark spec's tolerance and the
fp32 regression bound, and the arrival counters in the workspace must come back to zero so that
the next step can use the same workspace.
"""
import numpy as np
import pytest
import torch

from oracle import gh_oracle as O
from paper_2501_11779_amd import binding as G
from paper_2501_11779_amd import workloads as W
from tests import helpers as Hh

pytestmark = pytest.mark.gpu
DEV = "cuda"
KERNELS = {"valu": G.GH_KERNEL_VALU, "mfma": G.GH_KERNEL_MFMA}
RAGGED = np.array([0, 1, 31, 32, 33, 63, 64, 65, 127, 128, 129, 200, 255, 256, 257, 300, 511, 512,
                   513, 700], dtype=np.int32)


def step_workspace(p):
    """Workspace full of NaN (a record the kernel forgets poisons the result), counters cleared."""
    ws = G.alloc_workspace(p, DEV)
    ws.fill_(float("nan"))
    G.check(G.gh_decode_step_init(p, ws))
    return ws


def counters(p, ws):
    w = p.batch * p.n_q_heads
    return ws.view(torch.int32)[-w:].cpu().numpy()


def run_step(inp, chunk_rows=0, kernel=G.GH_KERNEL_AUTO, dtype=torch.float32, status=None, ws=None,
             max_ctx_len=None):
    p = G.problem_from_inputs(inp, chunk_rows=chunk_rows, kernel=kernel, max_ctx_len=max_ctx_len)
    w = inp["workload"]
    ws = step_workspace(p) if ws is None else ws
    out = torch.full((w.batch, w.n_q_heads, w.head_dim), float("nan"), dtype=dtype, device=DEV)
    G.decode_step_one_launch(p, inp, ws, out, dev_status=status)
    torch.cuda.synchronize()
    assert not counters(p, ws).any(), "arrival counters not back to zero"
    return out, p, ws


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("H,Hkv", [(4, 4), (8, 2), (8, 1), (6, 2), (32, 2), (40, 2), (40, 1), (72, 1)])
def test_one_launch_step_matches_oracle_on_ragged_batch(H, Hkv, dtype):
    w = W.Workload("step", len(RAGGED), H, Hkv, 128, dtype, ("const", 0), 140 + H + Hkv)
    inp = W.make_inputs(w, DEV, lengths=RAGGED, n_slots=len(RAGGED) + 3)
    host = Hh.host_copy(inp)
    out, _, _ = run_step(inp)
    want = Hh.oracle_step(inp, host)
    got = out.cpu().numpy()
    Hh.assert_parity(got, want, f"step {dtype} H={H}/{Hkv}")
    Hh.assert_tight(got, want, f"step {dtype} H={H}/{Hkv}")
    assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])      # the append, bit for bit
    assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])


@pytest.mark.parametrize("B,L", [(1, 5000), (1, 0), (2, 33000), (3, 257), (7, 1500), (40, 900)])
def test_small_batches_split_every_context_over_many_waves(B, L):
    """Few sequences: each context is cut into many pieces whose records the last wave merges
    (up to 64 per head), two at a time."""
    lengths = np.full(B, L, dtype=np.int32)
    lengths[0] = max(0, L - 7)
    w = W.Workload("stepsmall", B, 16, 2, 128, "bf16", ("const", 0), 150 + B)
    inp = W.make_inputs(w, DEV, lengths=lengths)
    host = Hh.host_copy(inp)
    out, p, _ = run_step(inp)
    want = Hh.oracle_step(inp, host)
    got = out.cpu().numpy()
    print(f"B={B} L={L}: records per head up to {G.gh_decode_num_chunks(p)}, "
          f"max_abs={np.abs(got - want).max():.2e}", flush=True)
    Hh.assert_tight(got, want, f"B={B} L={L}")
    assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])
    assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])


def test_decode_loop_reuses_one_workspace():
    """Five tokens generated one after the other with the same workspace: every step's counters
    are back at zero for the next, positions advance, the new rows of earlier steps are attended."""
    lengths = np.array([30, 31, 32, 0, 255, 700], dtype=np.int32)
    w = W.Workload("steploop", len(lengths), 8, 2, 128, "f16", ("const", 0), 160)
    inp = W.make_inputs(w, DEV, lengths=lengths, capacity=720)
    host = Hh.host_copy(inp)
    ws = None
    gen = torch.Generator(device=DEV)
    gen.manual_seed(5)
    for t in range(5):
        pos = lengths + t
        for name in ("q", "k_new", "v_new"):
            inp[name] = torch.randn(inp[name].shape, generator=gen, device=DEV).to(inp[name].dtype)
            host[name] = W.bits(inp[name])
        inp["pos"] = torch.from_numpy(pos.copy()).to(DEV)
        inp["ctx_len"] = (inp["pos"] + 1).to(torch.int32)
        host["pos"], host["ctx_len"] = pos.copy(), (pos + 1).astype(np.int32)
        inp["lengths"] = pos
        out, _, ws = run_step(inp, ws=ws, max_ctx_len=720)
        want = Hh.oracle_step(inp, host)
        Hh.assert_tight(out.cpu().numpy(), want, f"token {t}")
        assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])
        assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])


def test_bad_slot_or_position_is_skipped_flagged_and_leaves_the_rest_alone():
    lengths = np.array([100, 40, 7, 300, 64], dtype=np.int32)
    w = W.Workload("stepbad", 5, 8, 2, 128, "bf16", ("const", 0), 161)
    inp = W.make_inputs(w, DEV, lengths=lengths, n_slots=6, capacity=320)
    host = Hh.host_copy(inp)
    inp["slot_id"][1] = 17                                   # no such slot
    inp["pos"][3] = 320                                      # beyond the slot
    good = np.array([0, 2, 4])
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    out, _, _ = run_step(inp, status=status)
    got = out.cpu().numpy()
    assert int(status.item()) == (G.GH_DEV_BAD_SLOT | G.GH_DEV_BAD_POS)
    assert not got[1].any() and not got[3].any()
    # the oracle on the good sequences alone; the skipped ones appended nothing
    sub = dict(host)
    for name in ("q", "k_new", "v_new", "slot_id", "pos", "ctx_len"):
        sub[name] = host[name][good]
    import dataclasses
    inp_good = dict(inp, workload=dataclasses.replace(w, batch=3))
    want = Hh.oracle_step(inp_good, sub)
    Hh.assert_tight(got[good], want, "good sequences")
    assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])
    assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])


@pytest.mark.parametrize("layout", ["token_major", "head_blocked"])
def test_one_launch_step_on_other_cache_layouts(layout):
    w = W.Workload("steplay", len(RAGGED), 8, 2, 128, "bf16", ("const", 0), 162)
    inp = W.make_inputs(w, DEV, lengths=RAGGED, layout=layout, block_rows=64)
    host = Hh.host_copy(inp)
    out, _, _ = run_step(inp)
    Hh.assert_tight(out.cpu().numpy(), Hh.oracle_step(inp, host), layout)
    assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])
    assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_one_launch_step_with_the_16_bit_result(dtype):
    w = W.Workload("step16", len(RAGGED), 8, 2, 128, dtype, ("const", 0), 163)
    inp = W.make_inputs(w, DEV, lengths=RAGGED)
    host = Hh.host_copy(inp)
    out, _, _ = run_step(inp, dtype=W.TORCH_DTYPE[dtype])
    want = Hh.oracle_step(inp, host)
    same = Hh.assert_rounded_within(W.bits(out), want, dtype, Hh.TIGHT_MAX_ABS, "16-bit step")
    assert same > 0.995


@pytest.mark.parametrize("how", ["fixed_split", "valu"])
def test_the_three_kernel_route_of_the_step_call_gives_the_same(how):
    """Where the one-launch kernel does not apply the call issues append, attention and merge."""
    w = W.Workload("stepfix", len(RAGGED), 8, 2, 128, "f16", ("const", 0), 165)
    inp = W.make_inputs(w, DEV, lengths=RAGGED)
    chunk_rows, kernel = (128, G.GH_KERNEL_MFMA) if how == "fixed_split" else (0, G.GH_KERNEL_VALU)
    host = Hh.host_copy(inp)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    out, p, _ = run_step(inp, chunk_rows, kernel, status=status)
    assert G.gh_decode_split_plan(p).balanced == 0 and int(status.item()) == 0
    Hh.assert_tight(out.cpu().numpy(), Hh.oracle_step(inp, host), how)
    assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])
    assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])


def test_one_launch_step_on_a_batch_of_more_than_one_slice():
    """4100 sequences: the one launch becomes two, the second on the last four sequences; a bad
    position in the second slice is skipped and flagged like anywhere else."""
    w = W.Workload("stepbig", 4100, 4, 2, 128, "bf16", ("uniform", 0, 40), 164)
    inp = W.make_inputs(w, DEV)
    inp["pos"][4098] = inp["capacity"] + 5
    inp["ctx_len"][4098] = 0                                 # (what the oracle attends for it)
    host = Hh.host_copy(inp)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    out, p, _ = run_step(inp, 0, G.GH_KERNEL_AUTO, status=status)
    plan = G.gh_decode_split_plan(p)
    assert plan.balanced == 1 and plan.groups_per_launch == 4096 and int(status.item()) == 2
    po = Hh.oracle_problem(inp)
    assert O.kv_append(po, host["k_cache"], host["v_cache"], host["k_new"], host["v_new"],
                       host["slot_id"], host["pos"]) == 1
    want = O.decode_attention(po, host["q"], host["k_cache"], host["v_cache"], host["slot_id"],
                              host["ctx_len"])
    got = out.cpu().numpy()
    assert not got[4098].any()
    Hh.assert_tight(got, want, "4100 sequences in one call")
    assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])
    assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])


@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("H,Hkv", [(4, 4), (8, 1), (6, 2), (40, 2)])
def test_step_with_a_workgroup_per_strip(H, Hkv, dtype):
    """GH_KERNEL_STRIPS: the four waves of a workgroup share a strip and merge on chip.  Same
    contract, no workspace traffic: the workspace (never initialised here) stays as it was."""
    w = W.Workload("strips", len(RAGGED), H, Hkv, 128, dtype, ("const", 0), 170 + H + Hkv)
    inp = W.make_inputs(w, DEV, lengths=RAGGED, n_slots=len(RAGGED) + 3)
    host = Hh.host_copy(inp)
    p = G.problem_from_inputs(inp, kernel=G.GH_KERNEL_STRIPS)
    ws = G.alloc_workspace(p, DEV)
    ws.view(torch.int32).fill_(0x7fc00123)                   # NaN patterns, counters included
    for out_dtype in (torch.float32, W.TORCH_DTYPE[dtype]):
        out = torch.full((w.batch, H, 128), float("nan"), dtype=out_dtype, device=DEV)
        G.decode_step_one_launch(p, inp, ws, out)
        torch.cuda.synchronize()
        if out_dtype == torch.float32:
            want = Hh.oracle_step(inp, host)
            Hh.assert_tight(out.cpu().numpy(), want, f"strips {dtype} H={H}/{Hkv}")
            assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])
            assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])
        else:
            assert Hh.assert_rounded_within(W.bits(out), want, dtype, Hh.TIGHT_MAX_ABS, "strips 16-bit") > 0.995
    assert (ws.view(torch.int32) == 0x7fc00123).all()


def test_strips_step_flags_bad_entries_and_handles_layouts_and_a_decode_loop():
    lengths = np.array([100, 40, 7, 300, 64, 0, 31], dtype=np.int32)
    w = W.Workload("stripsbad", 7, 16, 2, 128, "bf16", ("const", 0), 171)
    for layout in ("head_major", "token_major", "head_blocked"):
        inp = W.make_inputs(w, DEV, lengths=lengths, n_slots=9, capacity=320, layout=layout, block_rows=64)
        host = Hh.host_copy(inp)
        p = G.problem_from_inputs(inp, kernel=G.GH_KERNEL_STRIPS, max_ctx_len=320)
        ws = G.alloc_workspace(p, DEV)
        out = torch.full((7, 16, 128), float("nan"), dtype=torch.float32, device=DEV)
        gen = torch.Generator(device=DEV)
        gen.manual_seed(3)
        for t in range(3):                                   # three tokens, positions advancing
            pos = lengths + t
            for name in ("q", "k_new", "v_new"):
                inp[name] = torch.randn(inp[name].shape, generator=gen, device=DEV).to(inp[name].dtype)
                host[name] = W.bits(inp[name])
            inp["pos"] = torch.from_numpy(pos.copy()).to(DEV)
            host["pos"], host["ctx_len"] = pos.copy(), (pos + 1).astype(np.int32)
            G.decode_step_one_launch(p, inp, ws, out)
            torch.cuda.synchronize()
            Hh.assert_tight(out.cpu().numpy(), Hh.oracle_step(inp, host), f"{layout} token {t}")
            assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])
            assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])
    # a slot that does not exist, a position beyond the slot
    inp["slot_id"][1] = 17
    inp["pos"][3] = 320
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    before_k = W.bits(inp["k_cache"])
    G.decode_step_one_launch(p, inp, ws, out, dev_status=status)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert int(status.item()) == (G.GH_DEV_BAD_SLOT | G.GH_DEV_BAD_POS)
    assert not got[1].any() and not got[3].any() and np.isfinite(got).all()
    changed = (W.bits(inp["k_cache"]) != before_k)
    assert not changed[int(host["slot_id"][3])].any()        # nothing appended for the bad position


def test_one_launch_step_is_bit_reproducible():
    w = W.Workload("steprep", 50, 16, 2, 128, "bf16", ("uniform", 0, 3000), 166)
    inp = W.make_inputs(w, DEV)
    a, _, ws = run_step(inp)
    b, _, _ = run_step(inp, ws=ws)                           # same row appended again: same inputs
    assert torch.equal(a.view(torch.int32), b.view(torch.int32))


def test_one_launch_step_captured_in_a_hip_graph():
    """One kernel node; replayed with rewritten device arrays, eager work in between."""
    lengths = np.array([10, 100, 33, 64, 0, 511], dtype=np.int32)
    w = W.Workload("stepgraph", len(lengths), 8, 2, 128, "bf16", ("const", 0), 167)
    inp = W.make_inputs(w, DEV, lengths=lengths, capacity=640)
    host = Hh.host_copy(inp)
    p = G.problem_from_inputs(inp, max_ctx_len=640)
    ws = step_workspace(p)
    out = torch.full((w.batch, 8, 128), float("nan"), dtype=torch.float32, device=DEV)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                            # warm-up outside the capture
        G.decode_step_one_launch(p, inp, ws, out)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        G.decode_step_one_launch(p, inp, ws, out)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(9)
    for t in range(4):
        pos = lengths + t
        for name in ("q", "k_new", "v_new"):
            inp[name].copy_(torch.randn(inp[name].shape, generator=gen, device=DEV).to(inp[name].dtype))
            host[name] = W.bits(inp[name])
        inp["pos"].copy_(torch.from_numpy(pos.copy()).to(DEV))
        host["pos"], host["ctx_len"] = pos.copy(), (pos + 1).astype(np.int32)
        (torch.ones(1000, device=DEV) * 2).sum().item()      # eager work between replays
        graph.replay()
        torch.cuda.synchronize()
        want = Hh.oracle_step(inp, host)
        Hh.assert_tight(out.cpu().numpy(), want, f"replay {t}")
        assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])

"""GPU parity: every entry point of the C ABI against the CPU oracle on seeded inputs.

Every case compares the whole output element by element (the full-size workloads C2-C5 are in
tests/test_gpu_full_size.py).  Tolerance for attention: max-abs 2e-3 and relative L2 1e-3
(16-bit K/V, fp32 accumulation), plus tighter regression bounds where a test says so; the append
is compared bit for bit.
"""
import math

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


def small(name, B, H, Hkv, dtype, seed):
    return W.Workload(name, B, H, Hkv, 128, dtype, ("const", 0), seed)


def run_gpu(inp, chunk_rows=0, kernel=G.GH_KERNEL_AUTO, append=True, status=None):
    p = G.problem_from_inputs(inp, chunk_rows=chunk_rows, kernel=kernel)
    w = inp["workload"]
    ws = G.alloc_workspace(p, DEV)
    ws.fill_(float("nan"))          # a record the kernel forgets to write poisons the output
    out = torch.full((w.batch, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.float32,
                     device=DEV)
    G.decode_step(p, inp, ws, out, dev_status=status, append=append)
    torch.cuda.synchronize()
    return out.cpu().numpy(), p, ws


# ------------------------------------------------------------------ append
@pytest.mark.parametrize("layout", ["head_major", "token_major"])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_append_bit_exact_whole_cache(layout, dtype):
    w = small("app", 5, 8, 4, dtype, 31)
    L = np.array([0, 7, 63, 64, 129], dtype=np.int32)
    inp = W.make_inputs(w, DEV, lengths=L, n_slots=7, capacity=131, layout=layout)
    host = Hh.host_copy(inp)
    p = G.problem_from_inputs(inp)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    G.check(G.gh_kv_append(p, inp["k_cache"], inp["v_cache"], inp["k_new"], inp["v_new"],
                           inp["slot_id"], inp["pos"], status))
    torch.cuda.synchronize()
    po = Hh.oracle_problem(inp)
    assert O.kv_append(po, host["k_cache"], host["v_cache"], host["k_new"], host["v_new"],
                       host["slot_id"], host["pos"]) == 0
    assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])
    assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])
    assert status.item() == 0


def test_append_flags_and_skips_bad_slot_or_position():
    w = small("bad", 4, 4, 2, "bf16", 32)
    inp = W.make_inputs(w, DEV, lengths=np.array([3, 4, 5, 6], dtype=np.int32), n_slots=4,
                        capacity=8)
    inp["slot_id"][1] = 9           # no such slot
    inp["pos"][2] = 8               # one past the capacity
    host = Hh.host_copy(inp)
    p = G.problem_from_inputs(inp)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    G.check(G.gh_kv_append(p, inp["k_cache"], inp["v_cache"], inp["k_new"], inp["v_new"],
                           inp["slot_id"], inp["pos"], status))
    torch.cuda.synchronize()
    assert status.item() == (G.GH_DEV_BAD_SLOT | G.GH_DEV_BAD_POS)
    po = Hh.oracle_problem(inp)
    assert O.kv_append(po, host["k_cache"], host["v_cache"], host["k_new"], host["v_new"],
                       host["slot_id"], host["pos"]) == 2
    assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])
    assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])


# ------------------------------------------------------------------ attention, small, whole output
RAGGED = np.array([0, 1, 30, 31, 32, 62, 63, 64, 65, 127, 128, 191, 299, 512, 700], dtype=np.int32)


@pytest.mark.parametrize("kernel", ["valu", "mfma"])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
@pytest.mark.parametrize("H,Hkv", [(4, 4), (4, 2), (8, 2), (8, 1), (6, 2), (32, 2), (40, 2),
                                  (40, 1),    # 40 heads on one kv head: three passes, the last strip half empty
                                  (72, 1)])   # five passes: the fourth wave of the worker carries no column
@pytest.mark.parametrize("chunk_rows", [64, 192, 0])
def test_attention_matches_oracle_on_ragged_batch(kernel, dtype, H, Hkv, chunk_rows):
    w = small("rag", len(RAGGED), H, Hkv, dtype, 40 + H + Hkv)
    inp = W.make_inputs(w, DEV, lengths=RAGGED, n_slots=len(RAGGED) + 3)
    host = Hh.host_copy(inp)
    got, p, _ = run_gpu(inp, chunk_rows, KERNELS[kernel])
    want = Hh.oracle_step(inp, host)
    Hh.assert_parity(got, want, f"{kernel} {dtype} H={H}/{Hkv} chunk={chunk_rows}")
    Hh.assert_tight(got, want, f"{kernel} {dtype} H={H}/{Hkv} chunk={chunk_rows}")
    # and the cache after the step is the oracle's mirror, bit for bit
    assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])
    assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])


@pytest.mark.parametrize("kernel", ["valu", "mfma"])
def test_more_than_64_records_per_head(kernel):
    """Fixed split with 64-row chunks over 4300 rows: 68 records per head, merged 64 at a time."""
    w = small("many", 3, 4, 2, "bf16", 51)
    inp = W.make_inputs(w, DEV, lengths=np.array([4300, 90, 4160], dtype=np.int32))
    host = Hh.host_copy(inp)
    got, p, _ = run_gpu(inp, 64, KERNELS[kernel])
    assert G.gh_decode_num_chunks(p) == 68
    Hh.assert_parity(got, Hh.oracle_step(inp, host), "68 records")


@pytest.mark.parametrize("route", ["three_kernels", "one_launch", "strips", "valu"])
def test_one_very_long_context_in_a_small_batch(route):
    """300 000 rows for one sequence (9 376 tiles per strip) beside two short ones: the balanced
    split runs out of records per head (64), so its shares grow beyond an equal split (min_share)
    and most waves get nothing; the strip kernel walks 2 344 tiles per wave; the vector kernel
    merges its chunks 64 at a time."""
    lengths = np.array([300000, 77, 4097], dtype=np.int32)
    w = small("long", 3, 8, 2, "bf16", 57)
    inp = W.make_inputs(w, DEV, lengths=lengths)
    host = Hh.host_copy(inp)
    want = Hh.oracle_step(inp, host)
    if route in ("three_kernels", "valu"):
        kernel = G.GH_KERNEL_MFMA if route == "three_kernels" else G.GH_KERNEL_VALU
        got, p, _ = run_gpu(inp, 0, kernel)
        if route == "three_kernels":
            plan = G.gh_decode_split_plan(p)
            assert plan.balanced and plan.n_chunks == 64
            total = sum(-(-int(n + 1) // 32) for n in lengths) * w.n_kv_heads
            assert plan.min_share > -(-total // plan.n_workers)      # the record bound binds
    else:
        p = G.problem_from_inputs(inp, kernel=G.GH_KERNEL_STRIPS if route == "strips" else G.GH_KERNEL_AUTO)
        ws = G.alloc_step_workspace(p, DEV)
        out = torch.full((w.batch, w.n_q_heads, 128), float("nan"), dtype=torch.float32, device=DEV)
        G.decode_step_one_launch(p, inp, ws, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
    Hh.assert_parity(got, want, f"long context, {route}")
    Hh.assert_tight(got, want, f"long context, {route}")
    assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])
    assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])


def test_largest_batch_of_the_balanced_split():
    """4096 sequences: the per-sequence arrays fill the kernel's dynamic LDS to its limit."""
    B = 4096
    w = W.Workload("lim", B, 4, 2, 128, "bf16", ("uniform", 0, 120), 53)
    inp = W.make_inputs(w, DEV)
    host = Hh.host_copy(inp)
    got, p, _ = run_gpu(inp, 0, G.GH_KERNEL_MFMA)
    assert G.gh_decode_chunk_rows(p) == 0
    Hh.assert_parity(got, Hh.oracle_step(inp, host), "B=4096")


@pytest.mark.parametrize("kernel", ["valu", "mfma"])
def test_rows_padded_to_twice_the_head_dim(kernel):
    """Explicit strides: each cached row sits in a 256-element pitch, slots are padded too."""
    B, H, Hkv, d, cap, n_slots, pitch = 5, 8, 2, 128, 300, 6, 256
    L = np.array([0, 100, 299, 64, 33], dtype=np.int32)
    w = small("pitch", B, H, Hkv, "bf16", 54)
    inp = W.make_inputs(w, DEV, lengths=L, n_slots=n_slots, capacity=cap)
    slot_pitch = Hkv * cap * pitch + 1024                      # padding between slots as well
    def widen(cache):
        flat = torch.full((n_slots * slot_pitch,), float("nan"), dtype=cache.dtype, device=DEV)
        view = flat.as_strided((n_slots, Hkv, cap, d), (slot_pitch, cap * pitch, pitch, 1))
        view.copy_(cache)
        return flat
    wide = dict(inp)
    wide["k_cache"], wide["v_cache"] = widen(inp["k_cache"]), widen(inp["v_cache"])
    wide["strides"] = (slot_pitch, cap * pitch, pitch)
    host = Hh.host_copy(wide)
    got, _, _ = run_gpu(wide, 64 if kernel == "valu" else 0, KERNELS[kernel])
    po = O.make_problem(B, H, Hkv, d, O.BF16, n_slots, cap, inp["scale"], wide["strides"])
    assert O.kv_append(po, host["k_cache"], host["v_cache"], host["k_new"], host["v_new"],
                       host["slot_id"], host["pos"]) == 0
    want = O.decode_attention(po, host["q"], host["k_cache"], host["v_cache"], host["slot_id"],
                              host["ctx_len"])
    Hh.assert_parity(got, want, "pitched rows")
    assert np.array_equal(W.bits(wide["k_cache"]), host["k_cache"])   # padding untouched, rows exact
    assert np.array_equal(W.bits(wide["v_cache"]), host["v_cache"])


@pytest.mark.parametrize("B", [4100, 8200])
def test_batch_above_one_launch_of_the_balanced_split_goes_in_slices(B):
    """More than 4096 sequences: the balanced split is launched on slices of 4096, each split on
    its own (a slice of four sequences; two full slices and a short one)."""
    w = W.Workload("big", B, 4, 2, 128, "f16", ("uniform", 0, 150), 52)
    inp = W.make_inputs(w, DEV)
    host = Hh.host_copy(inp)
    got, p, _ = run_gpu(inp, 0, G.GH_KERNEL_MFMA)
    plan = G.gh_decode_split_plan(p)
    assert G.gh_decode_chunk_rows(p) == 0 and plan.balanced == 1 and plan.groups_per_launch == 4096
    Hh.assert_tight(got, Hh.oracle_step(inp, host), f"B={B}")


def test_token_groups_above_one_launch_go_in_slices():
    """4100 groups of two tokens: the slices are cut at group borders."""
    T, groups = 2, 4100
    w = W.Workload("biggroups", groups * T, 4, 2, 128, "bf16", ("const", 0), 58)
    rng = np.random.default_rng(58)
    base = rng.integers(0, 60, size=groups)
    lengths = (np.repeat(base, T) + np.tile(np.arange(T), groups)).astype(np.int32)
    slots = np.repeat(rng.permutation(groups), T).astype(np.int32)
    inp = W.make_inputs(w, DEV, lengths=lengths, slots=slots, n_slots=groups)
    host = Hh.host_copy(inp)
    p = G.problem_from_inputs(inp, tokens_per_group=T)
    ws = G.alloc_workspace(p, DEV)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device=DEV)
    G.decode_step(p, inp, ws, out)
    torch.cuda.synchronize()
    assert G.gh_decode_split_plan(p).groups_per_launch == 4096
    Hh.assert_tight(out.cpu().numpy(), Hh.oracle_step(inp, host), "4100 groups")


@pytest.mark.parametrize("kernel", ["valu", "mfma"])
def test_token_major_layout(kernel):
    w = small("tok", 6, 8, 2, "bf16", 50)
    L = np.array([5, 64, 100, 257, 31, 400], dtype=np.int32)
    inp = W.make_inputs(w, DEV, lengths=L, layout="token_major")
    host = Hh.host_copy(inp)
    got, _, _ = run_gpu(inp, 128, KERNELS[kernel])
    Hh.assert_parity(got, Hh.oracle_step(inp, host), "token-major")


@pytest.mark.parametrize("chunk_rows", [0, 128])
@pytest.mark.parametrize("block_rows", [32, 256])
@pytest.mark.parametrize("kernel", ["valu", "mfma"])
def test_head_blocked_layout(kernel, block_rows, chunk_rows):
    """[slot][block][kv head][row][d]: lengths on, just before and just after block borders; the
    step's append must land in the right block as well (checked bit for bit on the whole cache)."""
    w = small("blk", 8, 8, 2, "bf16", 53)
    L = np.array([0, 31, 32, 255, 256, 257, 600, 1023], dtype=np.int32)
    inp = W.make_inputs(w, DEV, lengths=L, n_slots=9, layout="head_blocked", block_rows=block_rows)
    assert inp["capacity"] == 1024
    host = Hh.host_copy(inp)
    got, _, _ = run_gpu(inp, chunk_rows, KERNELS[kernel])
    Hh.assert_parity(got, Hh.oracle_step(inp, host), "head-blocked")
    assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])
    assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])


@pytest.mark.parametrize("kernel", ["valu", "mfma"])
def test_config1_whole_output(kernel):
    """C1 in full, at the benchmark spec's tolerance and at the regression bound of the fp32 path."""
    inp = W.make_inputs(W.WORKLOADS["c1"], DEV)
    host = Hh.host_copy(inp)
    got, _, _ = run_gpu(inp, 0, KERNELS[kernel])
    want = Hh.oracle_step(inp, host)
    Hh.assert_parity(got, want, "c1")
    Hh.assert_tight(got, want, "c1")
    assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])
    assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])


# ------------------------------------------------------------------ closed forms on the GPU
@pytest.mark.parametrize("kernel", ["valu", "mfma"])
@pytest.mark.parametrize("dtype", ["f16", "bf16"])
def test_length_one_returns_the_value_row_exactly(kernel, dtype):
    w = small("one", 3, 8, 2, dtype, 60)
    inp = W.make_inputs(w, DEV, lengths=np.zeros(3, dtype=np.int32), capacity=4)
    got, _, _ = run_gpu(inp, 0, KERNELS[kernel])
    v_new = inp["v_new"].float().cpu().numpy()            # exact widening of the appended row
    for h in range(8):
        assert np.array_equal(got[:, h], v_new[:, h // 4])


@pytest.mark.parametrize("kernel", ["valu", "mfma"])
def test_identical_keys_give_mean_of_values(kernel):
    w = small("mean", 2, 8, 2, "bf16", 61)
    L = np.array([200, 77], dtype=np.int32)
    inp = W.make_inputs(w, DEV, lengths=L, poison=False)
    inp["k_cache"][:] = inp["k_cache"][:, :, :1, :]
    inp["k_new"][:] = inp["k_cache"][inp["slot_id"].long(), :, 0, :]
    got, _, _ = run_gpu(inp, 64, KERNELS[kernel])
    v = inp["v_cache"].double().cpu().numpy()
    for b in range(2):
        n = L[b] + 1
        for h in range(8):
            want = v[inp["slots"][b], h // 4, :n].mean(axis=0)
            assert np.abs(got[b, h] - want).max() < 5e-6


@pytest.mark.parametrize("kernel", ["valu", "mfma"])
def test_one_hot_row_with_huge_score_is_finite_and_selected(kernel):
    w = small("hot", 1, 8, 1, "bf16", 62)
    inp = W.make_inputs(w, DEV, lengths=np.array([300], dtype=np.int32))
    # key row 123 = 4*q of head 0 would give a score of ~4*128/sqrt(128)=45 for that head
    inp["k_cache"][inp["slots"][0], 0, 123] = inp["q"][0, 0] * 4
    host = Hh.host_copy(inp)
    got, _, _ = run_gpu(inp, 64, KERNELS[kernel])
    want = Hh.oracle_step(inp, host)
    Hh.assert_parity(got, want, "one-hot")
    v123 = inp["v_cache"][inp["slots"][0], 0, 123].float().cpu().numpy()
    assert np.abs(got[0, 0] - v123).max() < 1e-3


# ------------------------------------------------------------------ robustness
@pytest.mark.parametrize("kernel", ["valu", "mfma"])
def test_zero_length_and_bad_slot_give_zeros_and_do_not_disturb_others(kernel):
    w = small("zero", 4, 8, 2, "bf16", 63)
    L = np.array([100, 50, 70, 20], dtype=np.int32)
    inp = W.make_inputs(w, DEV, lengths=L, n_slots=6)
    host = Hh.host_copy(inp)
    ref, _, _ = run_gpu(inp, 64, KERNELS[kernel])
    want = Hh.oracle_step(inp, host)
    Hh.assert_parity(ref, want, "baseline")
    inp["ctx_len"][1] = 0
    inp["slot_id"][2] = 77
    got, _, _ = run_gpu(inp, 64, KERNELS[kernel], append=False)
    assert not got[1].any() and not got[2].any()
    assert np.array_equal(got[0], ref[0]) and np.array_equal(got[3], ref[3])


@pytest.mark.parametrize("kernel", ["valu", "mfma"])
def test_bit_reproducible_and_batch_independent(kernel):
    w = small("rep", 8, 16, 4, "f16", 64)
    L = np.array([10, 900, 33, 257, 64, 511, 128, 700], dtype=np.int32)
    inp = W.make_inputs(w, DEV, lengths=L)
    a, _, _ = run_gpu(inp, 128, KERNELS[kernel])
    b, _, _ = run_gpu(inp, 128, KERNELS[kernel], append=False)
    assert np.array_equal(a, b)
    # the same sequence alone in a batch of one gives the same bits
    p1 = G.make_problem(1, 16, 4, 128, G.GH_F16, inp["n_slots"], inp["capacity"],
                        int(L.max()) + 1, inp["strides"], inp["scale"], 128, KERNELS[kernel])
    ws = G.alloc_workspace(p1, DEV)
    out = torch.empty((1, 16, 128), dtype=torch.float32, device=DEV)
    G.check(G.gh_decode_attention(p1, inp["q"][3:4].contiguous(), inp["k_cache"], inp["v_cache"],
                                  inp["slot_id"][3:4].contiguous(),
                                  inp["ctx_len"][3:4].contiguous(), ws))
    G.check(G.gh_decode_reduce(p1, ws, None, out))
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy()[0], a[3])


# ------------------------------------------------------------------ mixed prefill / decode batch
@pytest.mark.parametrize("kernel", ["valu", "mfma"])
@pytest.mark.parametrize("chunk_rows", [64, 0])
def test_mixed_prefill_and_decode_batch(kernel, chunk_rows):
    """Batch entries are tokens: prompt A adds a 37-token chunk to 100 cached rows, prompt C starts
    from an empty slot with 64 tokens, the rest are decode entries of other prompts."""
    lengths, slots = [], []
    lengths += [100 + t for t in range(37)]; slots += [2] * 37       # prefill chunk, prompt A
    lengths += [300, 31, 700]; slots += [0, 5, 6]                    # decode entries
    lengths += list(range(64)); slots += [3] * 64                    # fresh prompt C
    lengths += [257]; slots += [1]
    lengths, slots = np.array(lengths, dtype=np.int32), np.array(slots, dtype=np.int32)
    order = np.random.default_rng(3).permutation(len(lengths))        # entries in no special order
    lengths, slots = lengths[order], slots[order]
    w = small("mixed", len(lengths), 8, 2, "bf16", 68)
    inp = W.make_inputs(w, DEV, lengths=lengths, n_slots=8, capacity=704, slots=slots)
    host = Hh.host_copy(inp)
    got, _, _ = run_gpu(inp, chunk_rows, KERNELS[kernel])
    want = Hh.oracle_step(inp, host)
    Hh.assert_parity(got, want, "mixed batch")
    assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])
    assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])


# ------------------------------------------------------------------ token groups
def _grouped_rows(T):
    """Token rows in groups of T: chunks of two prompts, decode entries, padding.  Each row is
    (rows cached before it, slot, live); a padding row sits on a spare slot of its own."""
    spare = iter(range(10, 1000))
    rows = []

    def group(live_rows, pad_first=False):
        pad = [(0, next(spare), False) for _ in range(T - len(live_rows))]
        rows.extend(pad + live_rows if pad_first else live_rows + pad)

    def chunk(slot, cached, n_tokens):
        toks = [(cached + t, slot, True) for t in range(n_tokens)]
        for i in range(0, n_tokens, T):
            group(toks[i:i + T])

    chunk(2, 100, 2 * T + 2)                  # prompt A: a chunk over several groups, ragged end
    group([(300, 0, True)])                   # decode entries: one live row per group
    group([(31, 5, True)], pad_first=True)    # ... the live row need not come first
    group([])                                 # nothing live at all
    chunk(3, 0, T + 1)                        # prompt C starts from an empty slot
    group([(700, 6, True)])
    return rows


@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("H,Hkv,T", [(8, 1, 2), (8, 2, 4), (4, 4, 16), (8, 2, 3), (16, 2, 4),
                                     (6, 2, 5), (2, 2, 40),
                                     (8, 2, 12),     # 48 columns: two waves on one stream
                                     (16, 2, 16),    # 128 columns: four waves on one stream
                                     (10, 2, 16),    # 80 columns: five passes, the fourth wave has none
                                     (8, 1, 64)])    # 512 columns: four such strips
def test_token_groups_share_the_slot_stream_and_match_the_oracle(H, Hkv, T, dtype):
    """tokens_per_group = T: the T rows of a group are head columns of the same tiles, each masked
    at its own length.  The result must be the per-row oracle's (causal inside a chunk, zero for
    padding rows) and agree with the undeclared batch; appends are untouched."""
    rows = _grouped_rows(T)
    lengths = np.array([r[0] for r in rows], dtype=np.int32)
    slots = np.array([r[1] for r in rows], dtype=np.int32)
    live = np.array([r[2] for r in rows])
    w = small("groups", len(rows), H, Hkv, dtype, 69)
    inp = W.make_inputs(w, DEV, lengths=lengths, n_slots=int(slots.max()) + 1, capacity=704,
                        slots=slots)
    host = Hh.host_copy(inp)
    ctx = np.where(live, lengths + 1, 0).astype(np.int32)            # padding rows attend nothing
    inp["ctx_len"] = torch.from_numpy(ctx).to(DEV)
    host["ctx_len"] = ctx
    want = Hh.oracle_step(inp, host)
    assert not want[~live].any()

    outs = {}
    for tpg in (T, 0):
        p = G.problem_from_inputs(inp, tokens_per_group=tpg)
        ws = G.alloc_workspace(p, DEV)
        ws.fill_(float("nan"))
        out = torch.full((w.batch, H, 128), float("nan"), dtype=torch.float32, device=DEV)
        G.decode_step(p, inp, ws, out, append=(tpg == T))
        torch.cuda.synchronize()
        outs[tpg] = out.cpu().numpy()
        Hh.assert_parity(outs[tpg], want, f"tokens_per_group={tpg}")
    assert not outs[T][~live].any()
    assert np.abs(outs[T] - outs[0]).max() < 2e-5
    assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])
    assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])


def test_seeded_sweep_of_token_groups():
    """Thirty seeded batches of groups: random T, head counts and layouts; every group is a run of
    consecutive tokens of one prompt (possibly none, possibly not from the group's first row) with
    padding rows anywhere around it."""
    rng = np.random.default_rng(20250118)
    for case in range(30):
        T = int(rng.choice([2, 3, 4, 8, 16, 33, 64]))
        Hkv = int(rng.choice([1, 2, 4]))
        group = int(rng.choice([1, 2, 3, 4, 8, 16]))
        n_groups = int(rng.choice([1, 2, 5, 20]))
        layout = str(rng.choice(["head_major", "token_major", "head_blocked"]))
        dtype = str(rng.choice(["f16", "bf16"]))
        rows, spare = [], n_groups                       # prompt slots 0 .. n_groups-1, then spares
        for gidx in range(n_groups):
            k = int(rng.integers(0, T + 1))              # live tokens in this group
            first = int(rng.integers(0, T - k + 1))      # padding before them
            base = int(rng.choice([0, 1, 30, 31, 32, 100, 400]))
            for t in range(T):
                if first <= t < first + k:
                    rows.append((base + t - first, gidx, True))
                else:
                    rows.append((0, spare, False))
                    spare += 1
        lengths = np.array([r[0] for r in rows], dtype=np.int32)
        slots = np.array([r[1] for r in rows], dtype=np.int32)
        live = np.array([r[2] for r in rows])
        print(f"case {case}: T={T} Hkv={Hkv} group={group} groups={n_groups} {layout} {dtype} "
              f"rows={len(rows)} live={int(live.sum())}", flush=True)
        w = W.Workload(f"gsweep{case}", len(rows), Hkv * group, Hkv, 128, dtype, ("const", 0),
                       8000 + case)
        inp = W.make_inputs(w, DEV, lengths=lengths, n_slots=spare, capacity=448, slots=slots,
                            layout=layout, block_rows=64)
        host = Hh.host_copy(inp)
        ctx = np.where(live, lengths + 1, 0).astype(np.int32)
        inp["ctx_len"] = torch.from_numpy(ctx).to(DEV)
        host["ctx_len"] = ctx
        want = Hh.oracle_step(inp, host)
        p = G.problem_from_inputs(inp, tokens_per_group=T)
        ws = G.alloc_workspace(p, DEV)
        ws.fill_(float("nan"))
        out = torch.full((w.batch, Hkv * group, 128), float("nan"), dtype=torch.float32, device=DEV)
        G.decode_step(p, inp, ws, out)
        torch.cuda.synchronize()
        got = out.cpu().numpy()
        assert not got[~live].any()
        Hh.assert_parity(got, want, f"group sweep case {case}")
        assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])


@pytest.mark.parametrize("T", [4, 16])       # 16 columns per kv head; 64: a workgroup per worker
@pytest.mark.parametrize("layout", ["token_major", "head_blocked"])
def test_token_groups_on_other_cache_layouts(layout, T):
    """Grouping and addressing are independent: the same grouped batch on a token-major and on a
    head-blocked cache (blocks of 32 rows, so every chunk crosses block borders)."""
    rows = _grouped_rows(T)
    lengths = np.array([r[0] for r in rows], dtype=np.int32)
    slots = np.array([r[1] for r in rows], dtype=np.int32)
    live = np.array([r[2] for r in rows])
    w = small("groups2", len(rows), 8, 2, "bf16", 71)
    inp = W.make_inputs(w, DEV, lengths=lengths, n_slots=int(slots.max()) + 1, capacity=704,
                        slots=slots, layout=layout, block_rows=32)
    host = Hh.host_copy(inp)
    ctx = np.where(live, lengths + 1, 0).astype(np.int32)
    inp["ctx_len"] = torch.from_numpy(ctx).to(DEV)
    host["ctx_len"] = ctx
    want = Hh.oracle_step(inp, host)
    p = G.problem_from_inputs(inp, tokens_per_group=T)
    ws = G.alloc_workspace(p, DEV)
    ws.fill_(float("nan"))
    out = torch.full((w.batch, 8, 128), float("nan"), dtype=torch.float32, device=DEV)
    G.decode_step(p, inp, ws, out)
    torch.cuda.synchronize()
    Hh.assert_parity(out.cpu().numpy(), want, f"groups on {layout}")
    assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])


def test_token_group_row_on_another_slot_gets_no_rows():
    """A live row whose slot differs from that of the group's first live row is outside the
    declaration: it gets zeros, the rest of the group is unaffected."""
    lengths = np.array([50, 51, 40, 52], dtype=np.int32)
    slots = np.array([1, 1, 2, 1], dtype=np.int32)                   # row 2 breaks the group
    w = small("stray", 4, 8, 2, "bf16", 70)
    inp = W.make_inputs(w, DEV, lengths=lengths, n_slots=3, capacity=64, slots=slots)
    host = Hh.host_copy(inp)
    want = Hh.oracle_step(inp, host)
    p = G.problem_from_inputs(inp, tokens_per_group=4)
    ws = G.alloc_workspace(p, DEV)
    ws.fill_(float("nan"))
    out = torch.full((4, 8, 128), float("nan"), dtype=torch.float32, device=DEV)
    G.decode_step(p, inp, ws, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy()
    assert not got[2].any()
    Hh.assert_parity(got[[0, 1, 3]], want[[0, 1, 3]], "rest of the group")


# ------------------------------------------------------------------ the merge on its own
def test_reduce_matches_oracle_merge_of_oracle_partials():
    w = small("red", 3, 4, 2, "bf16", 65)
    L = np.array([300, 64, 5], dtype=np.int32)
    inp = W.make_inputs(w, "cpu", lengths=L)
    host = Hh.host_copy(inp)
    po = Hh.oracle_problem(inp)
    want = Hh.oracle_step(inp, host)
    chunk = 64
    p = G.problem_from_inputs(inp, chunk_rows=chunk)
    C_ = G.gh_decode_num_chunks(p)
    B, H, d = 3, 4, 128
    o = np.full((B, H, C_, d), np.nan, dtype=np.float32)
    m = np.full((B, H, C_), -np.inf, dtype=np.float32)
    l = np.zeros((B, H, C_), dtype=np.float32)
    for b in range(B):
        n = L[b] + 1
        for h in range(H):
            for c in range(C_):
                r0, r1 = c * chunk, min(n, (c + 1) * chunk)
                if r1 <= r0:
                    continue
                mm, ll, oo = O.partial(po, host["q"], host["k_cache"], host["v_cache"],
                                       host["slot_id"], b, h, r0, r1)
                m[b, h, c], l[b, h, c], o[b, h, c] = mm, ll, oo
    used = np.full((B, H), C_, dtype=np.int32)          # every record of every head is in use
    ws = torch.from_numpy(np.concatenate([o.ravel(), m.ravel(), l.ravel(),
                                          used.ravel().view(np.float32)])).to(DEV)
    out = torch.empty((B, H, d), dtype=torch.float32, device=DEV)
    G.check(G.gh_decode_reduce(p, ws, None, out))
    torch.cuda.synchronize()
    assert np.abs(out.cpu().numpy() - want).max() < 2e-6


@pytest.mark.parametrize("kernel", ["valu", "mfma"])
def test_attention_partials_match_oracle_partials(kernel):
    w = small("par", 2, 8, 2, "bf16", 66)
    L = np.array([200, 70], dtype=np.int32)
    inp = W.make_inputs(w, DEV, lengths=L)
    host = Hh.host_copy(inp)
    chunk = 64
    _, p, ws = run_gpu(inp, chunk, KERNELS[kernel])
    po = Hh.oracle_problem(inp)
    O.kv_append(po, host["k_cache"], host["v_cache"], host["k_new"], host["v_new"],
                host["slot_id"], host["pos"])
    C_ = G.gh_decode_num_chunks(p)
    B, H, d = 2, 8, 128
    wsn = ws.cpu().numpy()
    o = wsn[:B * H * C_ * d].reshape(B, H, C_, d)
    m = wsn[B * H * C_ * d:B * H * C_ * (d + 1)].reshape(B, H, C_)
    l = wsn[B * H * C_ * (d + 1):B * H * C_ * (d + 2)].reshape(B, H, C_)
    for b in range(B):
        n = L[b] + 1
        for h in range(H):
            for c in range(C_):
                r0, r1 = c * chunk, min(n, (c + 1) * chunk)
                if r1 <= r0:
                    assert m[b, h, c] == -np.inf and l[b, h, c] == 0.0
                    continue
                mm, ll, oo = O.partial(po, host["q"], host["k_cache"], host["v_cache"],
                                       host["slot_id"], b, h, r0, r1)
                # (m, l, o) is defined up to the common factor 2^m: compare what is unique
                assert abs((m[b, h, c] + math.log2(l[b, h, c])) - (mm + math.log2(ll))) < 1e-4
                assert np.abs(o[b, h, c] / l[b, h, c] - oo / ll).max() < Hh.MAX_ABS_TOL


def test_balanced_split_records_cover_each_head_exactly_once():
    """Library-chosen split: the records of a head are partial results over ranges the test does
    not know, so compare what is unique: their merged log-sum-exp and the count of live records."""
    w = small("bal", len(RAGGED), 8, 2, "bf16", 67)
    inp = W.make_inputs(w, DEV, lengths=RAGGED, n_slots=len(RAGGED) + 1)
    host = Hh.host_copy(inp)
    got, p, ws = run_gpu(inp, 0, G.GH_KERNEL_MFMA)
    assert G.gh_decode_chunk_rows(p) == 0
    Hh.assert_parity(got, Hh.oracle_step(inp, host), "balanced")
    po = Hh.oracle_problem(inp)
    C_ = G.gh_decode_num_chunks(p)
    B, H, d = len(RAGGED), 8, 128
    wsn = ws.cpu().numpy()
    m = wsn[B * H * C_ * d:B * H * C_ * (d + 1)].reshape(B, H, C_)
    l = wsn[B * H * C_ * (d + 1):B * H * C_ * (d + 2)].reshape(B, H, C_)
    used = wsn[B * H * C_ * (d + 2):B * H * C_ * (d + 2) + B * H].view(np.int32).reshape(B, H)
    assert used.min() >= 1 and used.max() <= C_
    for b in range(B):
        n = int(RAGGED[b]) + 1
        for h in range(H):
            live = np.arange(C_) < used[b, h]
            assert np.all(np.isfinite(l[b, h][live])) and np.all(l[b, h][live] > 0)
            lse = np.log2(np.sum(l[b, h][live].astype(np.float64) *
                                 np.exp2(m[b, h][live].astype(np.float64) - m[b, h][live].max()))) \
                + m[b, h][live].max()
            mm, ll, _ = O.partial(po, host["q"], host["k_cache"], host["v_cache"], host["slot_id"],
                                  b, h, 0, n)
            assert abs(lse - (mm + math.log2(ll))) < 1e-4


# ------------------------------------------------------------------ full-size workloads, sampled
# ------------------------------------------------------------------ ctx_len above the declared bound
@pytest.mark.parametrize("kernel", ["valu", "mfma"])
@pytest.mark.parametrize("chunk_rows", [0, 64])
def test_ctx_len_above_max_ctx_len_is_clamped_to_it(kernel, chunk_rows):
    """A ctx_len above min(max_ctx_len, slot_capacity) gives the result at that bound; the rows
    beyond it (NaN here) are never read."""
    lengths = np.array([99, 60, 2], dtype=np.int32)
    w = small("clamp", 3, 8, 2, "bf16", 77)
    inp = W.make_inputs(w, DEV, lengths=lengths, capacity=200)
    host = Hh.host_copy(inp)
    want = Hh.oracle_step(inp, host)                                  # ctx_len = 100, 61, 3
    inp["ctx_len"] = torch.tensor([150, 61, 3], dtype=torch.int32, device=DEV)
    p = G.problem_from_inputs(inp, chunk_rows=chunk_rows, kernel=KERNELS[kernel], max_ctx_len=100)
    ws = G.alloc_workspace(p, DEV)
    ws.fill_(float("nan"))
    out = torch.full((3, 8, 128), float("nan"), dtype=torch.float32, device=DEV)
    G.decode_step(p, inp, ws, out)
    torch.cuda.synchronize()
    Hh.assert_tight(out.cpu().numpy(), want, "clamped at max_ctx_len")
    # ... and at the slot capacity when that is the smaller bound
    inp2 = W.make_inputs(w, DEV, lengths=lengths, capacity=100)
    host2 = Hh.host_copy(inp2)
    want2 = Hh.oracle_step(inp2, host2)
    inp2["ctx_len"] = torch.tensor([100000, 61, 3], dtype=torch.int32, device=DEV)
    p2 = G.problem_from_inputs(inp2, chunk_rows=chunk_rows, kernel=KERNELS[kernel], max_ctx_len=100)
    ws2 = G.alloc_workspace(p2, DEV)
    out2 = torch.full((3, 8, 128), float("nan"), dtype=torch.float32, device=DEV)
    G.decode_step(p2, inp2, ws2, out2)
    torch.cuda.synchronize()
    Hh.assert_tight(out2.cpu().numpy(), want2, "clamped at the slot capacity")


# ------------------------------------------------------------------ seeded sweep of odd shapes
def test_seeded_sweep_of_shapes_layouts_and_splits():
    """Forty seeded cases that mix what the other tests vary one at a time: batch size, head-group
    size (up to two passes of 16 heads), length mixes with many empty and one-row sequences, spare
    slots, the three cache layouts, both kernels, both splits, both dtypes."""
    rng = np.random.default_rng(20250117)
    for case in range(40):
        B = int(rng.choice([1, 2, 3, 7, 33, 130, 300]))
        Hkv = int(rng.choice([1, 2, 4]))
        group = int(rng.choice([1, 2, 3, 4, 8, 16, 20, 32]))
        kind = rng.integers(0, 4)
        if kind == 0:
            L = rng.integers(0, 3, size=B)                       # empty and one-row contexts
        elif kind == 1:
            L = rng.integers(0, 200, size=B)
        elif kind == 2:
            L = np.where(rng.random(B) < 0.5, 0, rng.integers(0, 700, size=B))
        else:
            L = rng.integers(28, 36, size=B) * int(rng.integers(1, 12))   # around tile borders
        L = L.astype(np.int32)
        if B * Hkv * group * int(L.sum() + B) > 6_000_000:       # keep the oracle's work small
            L = (L // 4).astype(np.int32)
        layout = str(rng.choice(["head_major", "token_major", "head_blocked"]))
        kernel = str(rng.choice(["valu", "mfma"]))
        chunk_rows = int(rng.choice([0, 0, 64, 128]))
        dtype = str(rng.choice(["f16", "bf16"]))
        n_slots = B + int(rng.integers(0, 5))
        print(f"case {case}: B={B} Hkv={Hkv} group={group} kind={kind} max L={int(L.max())} "
              f"{layout} {kernel} chunk_rows={chunk_rows} {dtype} n_slots={n_slots}", flush=True)
        w = W.Workload(f"sweep{case}", B, Hkv * group, Hkv, 128, dtype, ("const", 0), 7000 + case)
        inp = W.make_inputs(w, DEV, lengths=L, n_slots=n_slots, layout=layout, block_rows=32)
        host = Hh.host_copy(inp)
        got, _, _ = run_gpu(inp, chunk_rows, KERNELS[kernel])
        want = Hh.oracle_step(inp, host)
        Hh.assert_parity(got, want, f"sweep case {case}")
        Hh.assert_tight(got, want, f"sweep case {case}")
        assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])
        assert np.array_equal(W.bits(inp["v_cache"]), host["v_cache"])


# ------------------------------------------------------------------ heads finished by the attention kernel
@pytest.mark.parametrize("native", [False, True])
@pytest.mark.parametrize("case", ["ragged", "groups", "large", "wide_groups", "many_heads"])
def test_attention_out_plus_merge_is_bit_identical_to_attention_plus_merge(case, native):
    """gh_decode_attention_out stores the heads one wave covers alone and marks them; the merge
    completes the rest.  The pair must give the same bits as attention + merge, in fp32 and in the
    16-bit type, and must really have finished heads early where strips are short."""
    tpg = 0
    if case == "ragged":
        w = small("early", 40, 8, 2, "bf16", 93)
        L = np.random.default_rng(5).integers(0, 500, size=40).astype(np.int32)
        L[:3] = [0, 31, 32]
        inp = W.make_inputs(w, DEV, lengths=L)
        ctx = None
    elif case in ("groups", "wide_groups"):
        # 4 tokens x 8 heads: 32 head columns, two passes per wave; 16 tokens: 128 columns, a
        # workgroup per worker (its own stores of records and final rows)
        tpg = 4 if case == "groups" else 16
        rows = _grouped_rows(tpg)
        L = np.array([r[0] for r in rows], dtype=np.int32)
        slots = np.array([r[1] for r in rows], dtype=np.int32)
        live = np.array([r[2] for r in rows])
        w = small("earlyg", len(rows), 16, 2, "f16", 94)
        inp = W.make_inputs(w, DEV, lengths=L, n_slots=int(slots.max()) + 1, capacity=704, slots=slots)
        ctx = np.where(live, L + 1, 0).astype(np.int32)
    elif case == "many_heads":
        w = small("earlyh", 40, 72, 1, "bf16", 96)                    # five passes on one kv head
        L = np.random.default_rng(6).integers(0, 500, size=40).astype(np.int32)
        inp = W.make_inputs(w, DEV, lengths=L)
        ctx = None
    else:
        w = W.Workload("earlyl", 1500, 8, 2, 128, "bf16", ("uniform", 0, 300), 95)   # many short strips
        inp = W.make_inputs(w, DEV)
        ctx = None
    host = Hh.host_copy(inp)
    if ctx is not None:
        inp["ctx_len"] = torch.from_numpy(ctx).to(DEV)
        host["ctx_len"] = ctx
    p = G.problem_from_inputs(inp, tokens_per_group=tpg)
    dt = W.TORCH_DTYPE[w.dtype] if native else torch.float32
    outs = []
    for early in (False, True):
        ws = G.alloc_workspace(p, DEV)
        ws.fill_(float("nan"))
        out = torch.full((w.batch, w.n_q_heads, 128), float("nan"), dtype=dt, device=DEV)
        G.decode_step(p, inp, ws, out, append=not early, early=early)
        torch.cuda.synchronize()
        outs.append(out)
        n_rec = Hh.record_counts(ws, w.batch, w.n_q_heads)
        if early:
            assert (n_rec == -1).mean() > (0.5 if case == "large" else 0.0)
        else:
            assert (n_rec >= 0).all()
    a, b = outs[0].cpu(), outs[1].cpu()
    assert torch.equal(a.view(torch.int32 if not native else torch.int16),
                       b.view(torch.int32 if not native else torch.int16))
    if not native:
        Hh.assert_parity(b.numpy(), Hh.oracle_step(inp, host), f"early {case}")


# ------------------------------------------------------------------ explicit streams
def test_step_on_an_explicit_stream_while_another_stream_is_busy():
    """Every call takes the stream it is given: a step issued on a side stream (default priority)
    while the current stream grinds through unrelated work, then awaited, matches the oracle."""
    w = small("stream", 5, 8, 2, "bf16", 92)
    L = np.array([10, 200, 31, 64, 333], dtype=np.int32)
    inp = W.make_inputs(w, DEV, lengths=L)
    host = Hh.host_copy(inp)
    p = G.problem_from_inputs(inp)
    ws = G.alloc_workspace(p, DEV)
    out = torch.full((w.batch, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.float32, device=DEV)
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    busy = torch.randn((2048, 2048), device=DEV)
    for _ in range(20):
        busy = busy @ busy.T * 1e-3                      # keeps the current stream occupied
    G.decode_step(p, inp, ws, out, stream=side)
    side.synchronize()
    Hh.assert_parity(out.cpu().numpy(), Hh.oracle_step(inp, host), "side stream")
    torch.cuda.synchronize()
    assert torch.isfinite(busy).all()


# ------------------------------------------------------------------ HIP graph replay
@pytest.mark.parametrize("kernel", ["valu", "mfma"])
def test_step_captured_in_a_hip_graph_replays_with_new_inputs(kernel):
    """The three calls only launch kernels, and everything that changes from token to token
    (lengths, positions, q, the new rows) lives in device arrays: a step captured once must give
    the oracle's result on every replay after those arrays were rewritten in place.  Eager work
    (poisoning the workspace and the output) and synchronisation sit between the replays."""
    w = small("graph", 6, 8, 2, "bf16", 90)
    L = np.array([0, 30, 31, 95, 200, 333], dtype=np.int32)
    inp = W.make_inputs(w, DEV, lengths=L, n_slots=7, capacity=400)
    host = Hh.host_copy(inp)
    p = G.problem_from_inputs(inp, max_ctx_len=400, kernel=KERNELS[kernel])
    ws = G.alloc_workspace(p, DEV)
    out = torch.empty((w.batch, w.n_q_heads, w.head_dim), dtype=torch.float32, device=DEV)
    status = torch.zeros(1, dtype=torch.int32, device=DEV)
    G.decode_step(p, inp, ws, out, dev_status=status)          # eager once: code objects are loaded
    torch.cuda.synchronize()
    Hh.assert_parity(out.cpu().numpy(), Hh.oracle_step(inp, host), "eager")

    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        G.decode_step(p, inp, ws, out, dev_status=status)
    gen = torch.Generator(device=DEV)
    gen.manual_seed(91)
    for replay in range(4):
        pos = L + 1 + 17 * replay                               # sequences grow by 17 rows a replay
        for name in ("q", "k_new", "v_new"):                   # new token, written in place
            inp[name].copy_(torch.randn(inp[name].shape, generator=gen, device=DEV).to(inp[name].dtype))
            host[name] = W.bits(inp[name])
        # rows [old length, pos) were never appended: give them values on both sides
        for b in range(w.batch):
            s, lo, hi = int(inp["slots"][b]), int(host["pos"][b]) + 1, int(pos[b])
            for which in ("k_cache", "v_cache"):
                fill = torch.randn((w.n_kv_heads, hi - lo, w.head_dim), generator=gen,
                                   device=DEV).to(inp[which].dtype)
                inp[which][s, :, lo:hi] = fill
                host[which][s, :, lo:hi] = W.bits(fill)
        inp["pos"].copy_(torch.from_numpy(pos.astype(np.int32)))
        inp["ctx_len"].copy_(torch.from_numpy((pos + 1).astype(np.int32)))
        host["pos"], host["ctx_len"] = pos.astype(np.int32), (pos + 1).astype(np.int32)
        ws.fill_(float("nan"))
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        Hh.assert_parity(out.cpu().numpy(), Hh.oracle_step(inp, host), f"replay {replay}")
        assert status.item() == 0
    assert np.array_equal(W.bits(inp["k_cache"]), host["k_cache"])


"""GPU parity at full size: the WHOLE output of workloads C2-C5 against the oracle.

Every sequence of every workload is recomputed by the float64 oracle (in slices of a few dozen
sequences, so the host never holds more than one slice of the cache) and compared element by
element with what the library produced in the launch configuration the benchmark times.  The
spec tolerance (max-abs 2e-3, relative L2 1e-3) is evaluated over the whole [B, H, d]
output, next to a much tighter regression bound on what the fp32 path really delivers; the
per-sequence worst case is printed.  After the step every slot of both caches must equal the
oracle's mirror bit for bit (the appended row and nothing else changed).

C4 and C5 are then rerun through the other ways a step can be launched -- heads finished by the
attention kernel, the 16-bit result, the paged slot pool with head-blocked pages -- against the
same oracle numbers.
"""
import numpy as np
import pytest
import torch

from oracle import gh_oracle as O
from paper_2501_11779_amd import binding as G
from paper_2501_11779_amd import workloads as W
from paper_2501_11779_amd.paged import into_pool, pages_needed
from tests import helpers as Hh

pytestmark = pytest.mark.gpu
DEV = "cuda"

SLICE = {"c2": 16, "c3": 64, "c4": 64, "c5": 4}     # sequences per oracle call
_WANT = {}                                           # (workload, layout) -> float64 [B, H, d]


def _slice_problem(inp, S):
    w = inp["workload"]
    strides = W.cache_shape_and_strides(S, w.n_kv_heads, inp["capacity"], w.head_dim,
                                        inp["layout"])[1]
    return O.make_problem(S, w.n_q_heads, w.n_kv_heads, w.head_dim, W.DTYPE_CODE[w.dtype], S,
                          inp["capacity"], inp["scale"], strides)


def _oracle_whole(inp, k_pre, v_pre, k_post=None, v_post=None):
    """Oracle append + attention over every sequence of `inp`, slice by slice, reading the
    pre-step caches `k_pre` / `v_pre` (device tensors indexed by slot).  With `k_post` / `v_post`
    (the caches after the library's step) each slice's mirror is compared with them bit for bit."""
    w = inp["workload"]
    B, step = w.batch, SLICE[w.name]
    want = np.empty((B, w.n_q_heads, w.head_dim), dtype=np.float64)
    for i in range(0, B, step):
        j = min(B, i + step)
        S = j - i
        slots = torch.from_numpy(inp["slots"][i:j].astype(np.int64)).to(DEV)
        kc, vc = W.bits(k_pre.index_select(0, slots)), W.bits(v_pre.index_select(0, slots))
        p = _slice_problem(inp, S)
        sid = np.arange(S, dtype=np.int32)
        pos = inp["lengths"][i:j].astype(np.int32)
        assert O.kv_append(p, kc, vc, W.bits(inp["k_new"][i:j]), W.bits(inp["v_new"][i:j]), sid,
                           pos) == 0
        want[i:j] = O.decode_attention(p, W.bits(inp["q"][i:j]), kc, vc, sid, pos + 1)
        if k_post is not None:
            assert np.array_equal(W.bits(k_post.index_select(0, slots)), kc), \
                f"{w.name}: K slots of sequences {i}..{j - 1} differ from the oracle's mirror"
            assert np.array_equal(W.bits(v_post.index_select(0, slots)), vc), \
                f"{w.name}: V slots of sequences {i}..{j - 1} differ from the oracle's mirror"
    return want


def _report(name, what, got, want, lengths):
    per_seq = np.abs(got - want).reshape(got.shape[0], -1).max(axis=1)
    b = int(per_seq.argmax())
    whole = Hh.assert_parity(got, want, f"{name} {what} whole output")
    print(f"{name} {what}: whole output max_abs={whole[0]:.2e} rel_l2={whole[1]:.2e}; worst "
          f"sequence {b} (len {int(lengths[b])}) max_abs={per_seq[b]:.2e}", flush=True)
    return whole


@pytest.mark.parametrize("name", ["c2", "c3", "c4", "c5"])
def test_whole_output_and_every_slot_at_full_size(name):
    w = W.WORKLOADS[name]
    inp = W.make_inputs(w, DEV)
    assert inp["n_slots"] == w.batch                       # every slot of the cache is compared
    k_pre, v_pre = inp["k_cache"].clone(), inp["v_cache"].clone()
    p = G.problem_from_inputs(inp)                         # the benchmark's launch configuration
    ws = G.alloc_workspace(p, DEV)
    ws.fill_(float("nan"))
    out = torch.full((w.batch, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.float32,
                     device=DEV)
    G.decode_step(p, inp, ws, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    want = _oracle_whole(inp, k_pre, v_pre, inp["k_cache"], inp["v_cache"])
    _WANT[(name, "head_major")] = want
    _report(name, "default launch", got, want, inp["lengths"])
    Hh.assert_tight(got, want, f"{name} default launch")


def _want_head_major(name, inp):
    key = (name, "head_major")
    if key not in _WANT:                                    # run alone: compute it here
        _WANT[key] = _oracle_whole(inp, inp["k_cache"], inp["v_cache"])
    return _WANT[key]


@pytest.mark.parametrize("name", ["c4", "c5"])
@pytest.mark.parametrize("variant", ["early", "out16", "early_out16"])
def test_whole_output_through_the_other_launch_paths(name, variant):
    w = W.WORKLOADS[name]
    inp = W.make_inputs(w, DEV)
    want = _want_head_major(name, inp)                      # from the caches before the step
    native = "out16" in variant
    p = G.problem_from_inputs(inp)
    ws = G.alloc_workspace(p, DEV)
    ws.fill_(float("nan"))
    dt = W.TORCH_DTYPE[w.dtype] if native else torch.float32
    out = torch.full((w.batch, w.n_q_heads, w.head_dim), float("nan"), dtype=dt, device=DEV)
    G.decode_step(p, inp, ws, out, early="early" in variant)
    torch.cuda.synchronize()
    if "early" in variant:
        n_rec = Hh.record_counts(ws, w.batch, w.n_q_heads)
        print(f"{name} {variant}: {(n_rec == -1).mean() * 100:.1f}% of the heads finished by the "
              f"attention kernel", flush=True)
    if not native:
        got = out.cpu().numpy().astype(np.float64)
        _report(name, variant, got, want, inp["lengths"])
        Hh.assert_tight(got, want, f"{name} {variant}")
        return
    # 16-bit result: the correct rounding of a value within the fp32 bound of the oracle's, and
    # nearly always the oracle's own value rounded once
    got_bits = W.bits(out)
    assert np.all(np.isfinite(W.from_bits(got_bits, w.dtype).float().numpy()))
    same = Hh.assert_rounded_within(got_bits, want, w.dtype, Hh.TIGHT_MAX_ABS, f"{name} {variant}")
    print(f"{name} {variant}: {same * 100:.3f}% of the 16-bit values identical to the rounded "
          f"oracle", flush=True)
    assert same > 0.995


@pytest.mark.parametrize("name", ["c2", "c4", "c5"])
def test_whole_output_of_the_one_launch_step(name):
    """gh_decode_step (append + attention + merge in one launch) at full size: the whole output
    against the oracle, the appended rows in place bit for bit and nothing else in the caches
    touched (the expectation for the caches is the pre-step copy with the new rows put in by
    plain indexing; the oracle's own mirror is compared in the three-call test above)."""
    w = W.WORKLOADS[name]
    inp = W.make_inputs(w, DEV)
    want = _want_head_major(name, inp)                      # from the caches before the step
    k_want, v_want = inp["k_cache"].clone(), inp["v_cache"].clone()
    slot, pos = inp["slot_id"].long(), inp["pos"].long()
    k_want[slot, :, pos] = inp["k_new"]
    v_want[slot, :, pos] = inp["v_new"]
    p = G.problem_from_inputs(inp)
    ws = G.alloc_workspace(p, DEV)
    ws.fill_(float("nan"))
    G.check(G.gh_decode_step_init(p, ws))
    out = torch.full((w.batch, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.float32,
                     device=DEV)
    G.decode_step_one_launch(p, inp, ws, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    _report(name, "one launch", got, want, inp["lengths"])
    Hh.assert_tight(got, want, f"{name} one launch")
    assert torch.equal(inp["k_cache"].view(torch.int16), k_want.view(torch.int16))
    assert torch.equal(inp["v_cache"].view(torch.int16), v_want.view(torch.int16))
    assert not ws.view(torch.int32)[-w.batch * w.n_q_heads:].any()      # arrival counters at zero


@pytest.mark.parametrize("name", ["c4", "c5"])
def test_whole_output_on_head_blocked_paged_slots(name):
    w = W.WORKLOADS[name]
    page_rows = 1024
    inp = W.make_inputs(w, DEV, layout="token_major")       # what into_pool() takes
    want = _oracle_whole(inp, inp["k_cache"], inp["v_cache"])
    need = pages_needed(inp["lengths"], page_rows)
    vcap = max(int(inp["lengths"].max()) + 1, int(3 * need * page_rows / w.batch))
    pool = G.SlotPool(inp["n_slots"], vcap, w.n_kv_heads, w.head_dim, page_rows, need,
                      layout="head_blocked")
    st = pool.stats()
    assert st.virtual_bytes / st.physical_bytes > 2.9        # oversubscribed as in the paper
    paged = into_pool(pool, inp)                             # NaN wherever nothing is cached
    del inp["k_cache"], inp["v_cache"]
    p = G.problem_from_inputs(paged)
    ws = G.alloc_workspace(p, DEV)
    ws.fill_(float("nan"))
    out = torch.full((w.batch, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.float32,
                     device=DEV)
    G.decode_step(p, paged, ws, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    _report(name, "head-blocked pages", got, want, paged["lengths"])
    Hh.assert_tight(got, want, f"{name} head-blocked pages")
    # the appended rows landed in the pages bit for bit
    dt = W.TORCH_DTYPE[w.dtype]
    for b in range(w.batch):
        s, n = int(paged["slots"][b]), int(paged["lengths"][b])
        for which, new in (("k", paged["k_new"]), ("v", paged["v_new"])):
            view = pool.rows_view(which, s, pool.mapped_rows(s), dt)
            row = view[n // page_rows, n % page_rows]          # [H_kv, d] of the appended row
            assert torch.equal(row.view(torch.int16), new[b].view(torch.int16)), (which, b)
    pool.close()


@pytest.mark.parametrize("name,T", [("c4", 16), ("c3", 16), ("c4", 4)])
def test_whole_output_of_prefill_chunks_at_full_size(name, T):
    """The workload's batch as B/T prefill chunks of T tokens, declared as token groups: chunks of 16
    at C4 shape are 128 head columns per kv head (a workgroup per worker, two passes per wave), at
    C3 shape 64 (one pass per wave), chunks of 4 at C4 shape 32 (two passes per wave).  Every entry
    against the oracle, which appends the whole batch and then lets entry t attend rows [0, pos_t]
    of its slot; the caches against the oracle's mirror, prompt by prompt."""
    base = W.WORKLOADS[name]
    prompts = base.batch // T
    lengths0 = W.draw_lengths(base)[:prompts]
    lengths = (np.repeat(lengths0, T) + np.tile(np.arange(T), prompts)).astype(np.int32)
    slots = np.repeat(np.arange(prompts), T).astype(np.int32)
    inp = W.make_inputs(base, DEV, lengths=lengths, slots=slots, n_slots=prompts)
    w = inp["workload"]
    k_pre, v_pre = inp["k_cache"].clone(), inp["v_cache"].clone()
    p = G.problem_from_inputs(inp, tokens_per_group=T)
    plan = G.gh_decode_split_plan(p)
    assert plan.waves_per_worker == (1 if T == 4 else 4)
    ws = G.alloc_workspace(p, DEV)
    ws.fill_(float("nan"))
    out = torch.full((w.batch, w.n_q_heads, w.head_dim), float("nan"), dtype=torch.float32,
                     device=DEV)
    G.decode_step(p, inp, ws, out)
    torch.cuda.synchronize()
    got = out.cpu().numpy().astype(np.float64)
    # the oracle, a few prompts at a time: each prompt's slot once, its T entries on it
    want = np.empty_like(got)
    per = max(1, 64 // T)
    for a in range(0, prompts, per):
        b = min(prompts, a + per)
        S, E = b - a, (b - a) * T
        rows = slice(a * T, b * T)
        sl = torch.arange(a, b, device=DEV)
        kc, vc = W.bits(k_pre.index_select(0, sl)), W.bits(v_pre.index_select(0, sl))
        strides = W.cache_shape_and_strides(S, w.n_kv_heads, inp["capacity"], w.head_dim,
                                            inp["layout"])[1]
        po = O.make_problem(E, w.n_q_heads, w.n_kv_heads, w.head_dim, W.DTYPE_CODE[w.dtype], S,
                            inp["capacity"], inp["scale"], strides)
        sid = np.repeat(np.arange(S), T).astype(np.int32)
        pos = lengths[rows]
        assert O.kv_append(po, kc, vc, W.bits(inp["k_new"][rows]), W.bits(inp["v_new"][rows]), sid,
                           pos) == 0
        want[rows] = O.decode_attention(po, W.bits(inp["q"][rows]), kc, vc, sid, pos + 1)
        assert np.array_equal(W.bits(inp["k_cache"].index_select(0, sl)), kc)
        assert np.array_equal(W.bits(inp["v_cache"].index_select(0, sl)), vc)
    _report(name, f"chunks of {T}", got, want, lengths)
    Hh.assert_tight(got, want, f"{name} chunks of {T}")

"""Host-side checks of the C ABI that need no GPU: exports, validation, chunk planning."""
import ctypes as C
import os
import re

import pytest

from paper_2501_11779_amd import binding as G

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_functions(header="gh_tier2.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(gh_[a-z_0-9]+)\s*\(", text)))


def good(**kw):
    base = dict(batch=4, n_q_heads=32, n_kv_heads=8, head_dim=128, dtype=G.GH_BF16, n_slots=4,
                slot_capacity=4097, max_ctx_len=4097, strides=(8 * 4097 * 128, 4097 * 128, 128),
                scale=128 ** -0.5, chunk_rows=0, kernel=G.GH_KERNEL_AUTO)
    base.update(kw)
    return G.make_problem(**base)


def test_library_loads_and_exports_every_declared_symbol():
    names = _declared_functions()
    assert set(names) == set(G.EXPORTS)
    L = G.lib()
    for n in names:
        assert getattr(L, n) is not None


def test_slot_pool_symbols_are_exported_and_arguments_checked_without_a_gpu():
    names = _declared_functions("gh_slot_pool.h")
    assert set(names) == set(G.POOL_EXPORTS)
    L = G.lib()
    for n in names:
        assert getattr(L, n) is not None
    handle = C.c_void_p()
    assert L.gh_slot_pool_create(None, C.byref(handle)) == G.GH_ERR_NULL
    cfg = G.gh_slot_pool_config(0, 100, 2, 128, 256, 0, 0, 4)
    assert L.gh_slot_pool_create(C.byref(cfg), C.byref(handle)) == G.GH_ERR_SHAPE
    cfg = G.gh_slot_pool_config(4, 100, 2, 64, 256, 0, 0, 4)
    assert L.gh_slot_pool_create(C.byref(cfg), C.byref(handle)) == G.GH_ERR_UNSUPPORTED
    cfg = G.gh_slot_pool_config(4, 100, 2, 128, 256, 0, 7, 4)                 # unknown layout
    assert L.gh_slot_pool_create(C.byref(cfg), C.byref(handle)) == G.GH_ERR_UNSUPPORTED
    cfg = G.gh_slot_pool_config(4, 100, 2, 128, 96, 0, G.GH_POOL_HEAD_BLOCKED, 4)
    assert L.gh_slot_pool_create(C.byref(cfg), C.byref(handle)) == G.GH_ERR_UNSUPPORTED
    assert L.gh_slot_pool_blocks(None, None, None) == G.GH_ERR_NULL
    assert L.gh_slot_pool_destroy(None) == G.GH_ERR_NULL
    assert L.gh_slot_pool_k(None) is None and L.gh_slot_pool_mapped_rows(None, 0) == 0
    assert L.gh_slot_pool_reserve(None, None, None, 0) == G.GH_ERR_NULL


def test_probe_symbol_is_exported_and_arguments_checked_without_a_gpu():
    assert _declared_functions("gh_probe.h") == ["gh_probe_stream_read"]
    a, MiB = 1 << 20, 1 << 20
    f = lambda *x: G.gh_probe_stream_read(*x, stream=0)
    assert f(None, 64 * MiB, 2048, 0, 0, None, a) == G.GH_ERR_NULL
    assert f(a, 64 * MiB, 2048, 4, 0, None, a) == G.GH_ERR_NULL               # stores need `rec`
    assert f(a, 64 * MiB, 2046, 0, 0, None, a) == G.GH_ERR_SHAPE              # waves in fours
    assert f(a, 64 * MiB + 4096, 2048, 0, 0, None, a) == G.GH_ERR_SHAPE       # whole tile pairs per wave
    assert f(a + 8, 64 * MiB, 2048, 0, 0, None, a) == G.GH_ERR_UNSUPPORTED
    assert f(a, 64 * MiB, 2048, 4, 9, a, a) == G.GH_ERR_UNSUPPORTED


def test_status_strings():
    for st in range(0, -8, -1):
        assert G.gh_status_string(st) not in ("", "unknown status")
    assert G.gh_status_string(-99) == "unknown status"


@pytest.mark.parametrize("kw,status", [
    (dict(n_kv_heads=5), G.GH_ERR_SHAPE),
    (dict(batch=-1), G.GH_ERR_SHAPE),
    (dict(n_slots=0), G.GH_ERR_SHAPE),
    (dict(head_dim=64), G.GH_ERR_UNSUPPORTED),
    (dict(dtype=7), G.GH_ERR_UNSUPPORTED),
    (dict(kernel=9), G.GH_ERR_UNSUPPORTED),
    (dict(strides=(8 * 4097 * 128, 4097 * 128, 64)), G.GH_ERR_SHAPE),
    (dict(strides=(8 * 4097 * 128 + 4, 4097 * 128, 128)), G.GH_ERR_UNSUPPORTED),
    (dict(max_ctx_len=5000), G.GH_ERR_CAPACITY),
    (dict(chunk_rows=100), G.GH_ERR_SHAPE),
    (dict(chunk_rows=-64), G.GH_ERR_SHAPE),
    (dict(q_batch_stride=32 * 128 - 8), G.GH_ERR_SHAPE),
    (dict(new_batch_stride=-8), G.GH_ERR_SHAPE),
    (dict(tokens_per_group=-1), G.GH_ERR_SHAPE),
    (dict(tokens_per_group=3), G.GH_ERR_SHAPE),                       # batch 4 is no multiple of 3
    (dict(tokens_per_group=2, kernel=G.GH_KERNEL_VALU), G.GH_ERR_UNSUPPORTED),
    (dict(tokens_per_group=2, chunk_rows=64), G.GH_ERR_UNSUPPORTED),
    (dict(tokens_per_group=65, batch=130), G.GH_ERR_UNSUPPORTED),
    (dict(block=(-32, 4096)), G.GH_ERR_SHAPE),
    (dict(block=(64, 0)), G.GH_ERR_SHAPE),
    (dict(block=(48, 8 * 48 * 128)), G.GH_ERR_UNSUPPORTED),
    (dict(block=(16, 8 * 16 * 128)), G.GH_ERR_UNSUPPORTED),
    (dict(block=(64, 8 * 64 * 128 + 4)), G.GH_ERR_UNSUPPORTED),
    (dict(q_batch_stride=48 * 128 + 4), G.GH_ERR_UNSUPPORTED),
])
def test_invalid_problems_are_refused_by_every_entry_point(kw, status):
    p = good(**kw)
    assert G.gh_decode_chunk_rows(p) == status
    assert G.gh_decode_num_chunks(p) == status
    assert G.gh_decode_workspace_bytes(p) == 0
    fake = 4096  # never dereferenced: validation fails first
    assert G.gh_kv_append(p, fake, fake, fake, fake, fake, fake, None, 0) == status
    assert G.gh_decode_attention(p, fake, fake, fake, fake, fake, fake, 1 << 40, 0) == status
    assert G.gh_decode_reduce(p, fake, None, fake, 0) == status
    assert G.gh_decode_reduce_native(p, fake, None, fake, 0) == status


def test_null_problem_and_null_pointers():
    L = G.lib()
    assert L.gh_decode_chunk_rows(None) == G.GH_ERR_NULL
    assert L.gh_kv_append(None, 1, 1, 1, 1, 1, 1, None, None) == G.GH_ERR_NULL
    p = good()
    a = 4096
    assert G.gh_kv_append(p, None, a, a, a, a, a, None, 0) == G.GH_ERR_NULL
    assert G.gh_kv_append(p, a, a, a, a, None, a, None, 0) == G.GH_ERR_NULL
    assert G.gh_decode_attention(p, a, a, a, a, None, a, 1 << 40, 0) == G.GH_ERR_NULL
    assert G.gh_decode_attention(p, a, a, a, a, a, None, 1 << 40, 0) == G.GH_ERR_NULL
    assert G.gh_decode_reduce(p, None, None, a, 0) == G.GH_ERR_NULL
    assert G.gh_decode_reduce(p, a, None, None, 0) == G.GH_ERR_NULL


def test_misaligned_pointers_and_small_workspace():
    p = good()
    a = 4096
    assert G.gh_kv_append(p, a + 2, a, a, a, a, a, None, 0) == G.GH_ERR_UNSUPPORTED
    assert G.gh_decode_attention(p, a + 8, a, a, a, a, a, 1 << 40, 0) == G.GH_ERR_UNSUPPORTED
    need = G.gh_decode_workspace_bytes(p)
    assert need > 0
    assert G.gh_decode_attention(p, a, a, a, a, a, a, need - 1, 0) == G.GH_ERR_WORKSPACE


def test_empty_batch_is_a_no_op():
    p = good(batch=0)
    assert G.gh_kv_append(p, None, None, None, None, None, None, None, 0) == G.GH_OK
    assert G.gh_decode_attention(p, None, None, None, None, None, None, 0, 0) == G.GH_OK
    assert G.gh_decode_reduce(p, None, None, None, 0) == G.GH_OK
    assert G.gh_decode_workspace_bytes(p) == 0


@pytest.mark.parametrize("kernel", [G.GH_KERNEL_AUTO, G.GH_KERNEL_VALU, G.GH_KERNEL_MFMA])
@pytest.mark.parametrize("B,H,Hkv,maxlen", [(4, 8, 8, 513), (64, 32, 32, 2049), (256, 32, 8, 4097),
                                           (1024, 64, 8, 4097), (32, 64, 8, 32769), (1, 1, 1, 1)])
def test_chunk_plan_is_consistent(kernel, B, H, Hkv, maxlen):
    p = good(batch=B, n_q_heads=H, n_kv_heads=Hkv, n_slots=B, slot_capacity=maxlen,
             max_ctx_len=maxlen, strides=(Hkv * maxlen * 128, maxlen * 128, 128), kernel=kernel)
    rows = G.gh_decode_chunk_rows(p)
    n = G.gh_decode_num_chunks(p)
    if kernel == G.GH_KERNEL_VALU:
        assert rows > 0 and rows % 64 == 0          # fixed split into chunks of `rows` rows
        assert n == -(-maxlen // rows) and n >= 1
    else:
        assert rows == 0                            # balanced split: equal shares per wave
        assert 2 <= n <= 64
    # o, m, l of every record; the record count and the arrival counter of every head
    assert G.gh_decode_workspace_bytes(p) == B * H * (n * (128 + 2) + 2) * 4
    # a forced chunk size is taken as given
    p.chunk_rows = 128
    assert G.gh_decode_chunk_rows(p) == 128
    assert G.gh_decode_num_chunks(p) == -(-maxlen // 128)


def test_problem_struct_matches_header_field_order():
    text = open(os.path.join(ROOT, "include", "gh_tier2.h")).read()
    body = re.search(r"typedef struct \{(.*?)\} gh_problem;", text, flags=re.S).group(1)
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    fields = []
    for decl in body.split(";"):
        decl = decl.strip()
        if not decl:
            continue
        ctype, names = decl.split(None, 1)
        fields += [(n.strip(), ctype) for n in names.split(",")]
    want = {"int32_t": C.c_int32, "int64_t": C.c_int64, "float": C.c_float}
    assert [(n, want[t]) for n, t in fields] == list(G.gh_problem._fields_)


# ------------------------------------------------------------------ the balanced split, emulated
def _emulate_balanced_split(plan, group_rows, n_kv_heads):
    """The split as include/gh_tier2.h words it, in plain Python: returns, per strip, the list of
    (record index, first tile, last tile + 1) pieces the waves write, in wave order."""
    strips_per_group = n_kv_heads * plan.strips_per_kv_head
    tiles = [max(1, -(-n // 32)) for n in group_rows]             # per strip of the group
    first_tile, t = [], 0                                          # of every strip, laid end to end
    for tl in tiles:
        for _ in range(strips_per_group):
            first_tile.append(t)
            t += tl
    total = t
    share = max(-(-total // plan.n_workers), plan.min_share)
    pieces = [[] for _ in first_tile]
    strip = 0
    for w in range(plan.n_workers):
        lo, hi = w * share, min((w + 1) * share, total)
        if lo >= total:
            break
        while strip + 1 < len(first_tile) and first_tile[strip + 1] <= lo:
            strip += 1
        s = strip
        while s < len(first_tile) and first_tile[s] < hi:
            n_tiles = tiles[s // strips_per_group]
            a, b = max(lo, first_tile[s]), min(hi, first_tile[s] + n_tiles)
            pieces[s].append((w - first_tile[s] // share, a - first_tile[s], b - first_tile[s]))
            s += 1
    return pieces, tiles, strips_per_group


@pytest.mark.parametrize("seed", range(12))
def test_balanced_split_never_needs_more_records_than_the_workspace_has(seed):
    """Safety of the record index: for lengths up to max_ctx_len, however uneven, every piece a wave
    writes has an index in [0, gh_decode_num_chunks), indices of a strip are consecutive from 0 and
    its pieces tile [0, tiles) in order.  (A larger index would be a write outside the workspace.)"""
    import numpy as np
    rng = np.random.default_rng(1000 + seed)
    for _ in range(25):
        T = int(rng.choice([1, 1, 1, 2, 4, 16]))
        groups = int(rng.choice([1, 2, 3, 17, 64, 300, 1024, 4096]))
        Hkv = int(rng.choice([1, 2, 8]))
        G_ = int(rng.choice([1, 4, 8, 20, 40]))
        max_ctx = int(rng.choice([1, 31, 32, 33, 100, 1000, 4097, 32769]))
        if groups * T > 8192:
            groups = 8192 // T
        p = good(batch=groups * T, n_q_heads=Hkv * G_, n_kv_heads=Hkv, n_slots=max(groups, 1),
                 slot_capacity=max_ctx, max_ctx_len=max_ctx,
                 strides=(Hkv * max_ctx * 128, max_ctx * 128, 128), tokens_per_group=T)
        plan = G.gh_decode_split_plan(p)
        assert plan.balanced == 1 and plan.n_chunks == G.gh_decode_num_chunks(p)
        kind = rng.integers(0, 5)
        if kind == 0:
            rows = np.full(groups, max_ctx)                       # everything at the limit
        elif kind == 1:
            rows = np.zeros(groups, dtype=np.int64)               # one long context among empty ones
            rows[rng.integers(0, groups)] = max_ctx
        elif kind == 2:
            rows = rng.integers(0, max_ctx + 1, size=groups)
        elif kind == 3:
            rows = np.where(rng.random(groups) < 0.9, rng.integers(0, 3, size=groups), max_ctx)
        else:
            rows = np.minimum(max_ctx, rng.geometric(1.0 / max(1, max_ctx // 8), size=groups))
        pieces, tiles, spg = _emulate_balanced_split(plan, [int(r) for r in rows], Hkv)
        for s, ps in enumerate(pieces):
            assert ps, "a strip nobody visits"
            assert [rec for rec, _, _ in ps] == list(range(len(ps)))
            assert len(ps) <= plan.n_chunks, (len(ps), plan.n_chunks, groups, Hkv, G_, T, max_ctx, kind)
            pos = 0
            for _, a, b in ps:
                assert a == pos and b > a
                pos = b
            assert pos == tiles[s // spg]


def test_split_plan_reports_the_fixed_split_and_checks_its_arguments():
    p = good(kernel=G.GH_KERNEL_VALU)
    plan = G.gh_decode_split_plan(p)
    assert plan.balanced == 0 and plan.n_workers == 0 and plan.n_chunks == G.gh_decode_num_chunks(p)
    assert G.lib().gh_decode_split_plan(C.byref(p), None) == G.GH_ERR_NULL
    assert G.lib().gh_decode_split_plan(None, C.byref(G.gh_split_plan())) == G.GH_ERR_NULL
    two = G.gh_decode_split_plan(good(n_q_heads=64, n_kv_heads=2, strides=(2 * 4097 * 128, 4097 * 128, 128)))
    assert two.passes_per_strip == 2 and two.strips_per_kv_head == 1 and two.n_workers == 1024
    assert two.waves_per_worker == 1
    # 16 tokens of 8 heads per kv head: 128 head columns = four waves of two passes on one stream
    four = G.gh_decode_split_plan(good(batch=64, tokens_per_group=16, n_q_heads=64, n_kv_heads=8))
    assert (four.passes_per_strip, four.waves_per_worker, four.strips_per_kv_head, four.n_workers) \
        == (2, 4, 1, 512)
    # 64 tokens: 512 columns = four such strips; 3 passes: four waves of one pass, the last without columns
    assert G.gh_decode_split_plan(good(batch=64, tokens_per_group=64, n_q_heads=64, n_kv_heads=8)
                                  ).strips_per_kv_head == 4
    assert four.groups_per_launch == 4                     # 64 entries are four groups of 16
    # a batch beyond one launch goes in slices of 4096 groups; the numbers are those of a slice
    big = G.gh_decode_split_plan(good(batch=10000, n_slots=10000))
    assert big.balanced == 1 and big.groups_per_launch == 4096
    assert big.n_chunks == G.gh_decode_split_plan(good(batch=4096, n_slots=4096)).n_chunks
    three = G.gh_decode_split_plan(good(n_q_heads=40, n_kv_heads=1, strides=(4097 * 128, 4097 * 128, 128)))
    assert (three.passes_per_strip, three.waves_per_worker, three.strips_per_kv_head, three.n_workers) \
        == (1, 4, 1, 512)


def test_public_headers_are_plain_c(tmp_path):
    """The boundary is a C ABI: every header under include/ must compile as strict C99 on its own
    (and as C++), with nothing but <stddef.h> / <stdint.h> behind it."""
    import shutil
    import subprocess
    inc = os.path.join(ROOT, "include")
    headers = sorted(f for f in os.listdir(inc) if f.endswith(".h"))
    assert headers == ["gh_probe.h", "gh_sim.h", "gh_slot_pool.h", "gh_tier2.h"]
    for h in headers:
        src = tmp_path / (h[:-2] + "_only.c")
        src.write_text(f'#include "{h}"\nint main(void) {{ return 0; }}\n')
        for cc, std in (("gcc", ["-std=c99", "-pedantic"]), ("g++", ["-std=c++11", "-x", "c++"])):
            if shutil.which(cc) is None:
                pytest.skip(f"{cc} not available")
            res = subprocess.run([cc, *std, "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", inc,
                                  str(src)], capture_output=True, text=True)
            assert res.returncode == 0, f"{h} with {cc}: {res.stderr}"


def test_step_call_checks_its_arguments():
    p = good()
    a, big = 4096, 1 << 40
    f = lambda *x: G.lib().gh_decode_step(C.byref(x[0]), *x[1:])
    args = [p, a, a, a, a, a, a, a, a, big, a, G.GH_OUT_F32, None, None]
    for missing in (1, 2, 3, 4, 5, 6, 7, 8, 10):
        bad = list(args)
        bad[missing] = None
        assert f(*bad) == G.GH_ERR_NULL, missing
    bad = list(args); bad[11] = 5
    assert f(*bad) == G.GH_ERR_UNSUPPORTED
    bad = list(args); bad[10] = a + 4
    assert f(*bad) == G.GH_ERR_UNSUPPORTED                        # out not 16-byte aligned
    bad = list(args); bad[9] = 64
    assert f(*bad) == G.GH_ERR_WORKSPACE
    grouped = good(tokens_per_group=2)
    assert f(grouped, *args[1:]) == G.GH_ERR_UNSUPPORTED
    assert G.lib().gh_decode_step_init(C.byref(p), None, big, None) == G.GH_ERR_NULL
    assert G.lib().gh_decode_step_init(C.byref(p), a, 64, None) == G.GH_ERR_WORKSPACE
    assert G.lib().gh_decode_step_init(C.byref(good(batch=0)), None, 0, None) == G.GH_OK


def test_attention_out_checks_its_arguments():
    p = good()
    a = 4096
    assert G.gh_decode_attention_out(p, a, a, a, a, a, a, None, G.GH_OUT_F32, 1 << 40, 0) == G.GH_ERR_NULL
    assert G.gh_decode_attention_out(p, a, a, a, a, a, a, a + 4, G.GH_OUT_F32, 1 << 40, 0) \
        == G.GH_ERR_UNSUPPORTED
    assert G.gh_decode_attention_out(p, a, a, a, a, a, a, a, 7, 1 << 40, 0) == G.GH_ERR_UNSUPPORTED
    assert G.gh_decode_attention_out(p, a, a, a, a, a, a, a, G.GH_OUT_NATIVE, 16, 0) == G.GH_ERR_WORKSPACE
    assert G.gh_decode_attention_out(good(batch=0), None, None, None, None, None, None, None,
                                     G.GH_OUT_F32, 0, 0) == G.GH_OK



# ------------------------------------------------------------------ slot pool bookkeeping, no GPU
def test_reserve_takes_back_what_it_mapped_when_the_runtime_refuses_a_page():
    """All or nothing also when the failure comes from the runtime in the middle of a request:
    a host-only pool whose 5th page mapping fails."""
    pool = G.SlotPool(6, 1000, 2, 128, 256, physical_pages=12, host_only_fail_at=4)
    assert pool.k_ptr is None and pool.capacity == 1024
    assert pool.reserve([0, 1], [512, 300]) == G.GH_OK                    # mappings 0-3
    assert pool.stats().pages_mapped == 4 and pool.stats().pages_created == 4
    before = [pool.mapped_rows(s) for s in range(6)]
    # needs 1 + 3 + 2 more pages; the first of them is the mapping that fails
    assert pool.reserve([0, 2, 3], [700, 768, 512]) == G.GH_ERR_HIP
    assert [pool.mapped_rows(s) for s in range(6)] == before
    st = pool.stats()
    assert st.pages_mapped == 4 and st.slots_in_use == 2 and st.pages_created == 5
    # ... and when it fails after some of the request went through (mapping 4 failed above, so
    # count on: a second pool that fails on its 7th)
    pool.close()
    pool = G.SlotPool(6, 1000, 2, 128, 256, physical_pages=12, host_only_fail_at=6)
    assert pool.reserve([0, 1], [512, 300]) == G.GH_OK                    # mappings 0-3
    before = [pool.mapped_rows(s) for s in range(6)]
    assert pool.reserve([0, 2, 3], [700, 768, 512]) == G.GH_ERR_HIP      # 4, 5 succeed, 6 fails
    assert [pool.mapped_rows(s) for s in range(6)] == before
    assert pool.stats().pages_mapped == 4
    # the pages taken back are usable: the same request now goes through (mappings 7-12)
    assert pool.reserve([0, 2, 3], [700, 768, 512]) == G.GH_OK
    assert [pool.mapped_rows(s) for s in range(6)] == [768, 512, 768, 512, 0, 0]
    assert pool.stats().pages_mapped == 10 and pool.stats().pages_created == 10
    # the budget still binds: 2 pages left, 3 wanted
    assert pool.reserve([4], [768]) == G.GH_ERR_CAPACITY
    assert pool.release([0, 1, 2, 3]) == G.GH_OK
    assert pool.stats().pages_mapped == 0 and pool.stats().pages_created == 10
    pool.close()


def test_host_only_pool_checks_its_configuration_like_the_real_one():
    with pytest.raises(G.GhError) as e:
        G.SlotPool(0, 100, 2, 128, 256, 4, host_only_fail_at=-1)
    assert e.value.status == G.GH_ERR_SHAPE
    with pytest.raises(G.GhError) as e:
        G.SlotPool(4, 100, 2, 128, 96, 4, layout="head_blocked", host_only_fail_at=-1)
    assert e.value.status == G.GH_ERR_UNSUPPORTED

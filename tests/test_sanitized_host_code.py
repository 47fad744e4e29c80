"""Host code under AddressSanitizer and UndefinedBehaviorSanitizer (CPU only, nothing on a GPU).

Three small drivers under tests/native/ are compiled with `-fsanitize=address,undefined` (runtimes
linked statically, so nothing has to be preloaded) and run as child processes:

  * oracle/gh_oracle.c on ragged batches in the three cache layouts, every array in a heap block of
    exactly its size: its results must be bit for bit those of the ordinary build that the parity
    tests use, and the sanitizers must stay silent;
  * the pipeline simulators of csrc/gh_sim.hip (plain host C++) on the sixty seeded configurations
    of tests/test_sim.py, token times equal to the Python oracle's to the last bit;
  * csrc/gh_plan.hpp: the balanced split replayed in C++ from the library's own planning code with
    the kernel's record arithmetic, checked against the Python emulation of the same split in
    tests/test_abi_host.py on seeded problems with adversarial length mixes.
"""
import os
import shutil
import struct
import subprocess

import numpy as np
import pytest

from oracle import gh_oracle as O
from oracle import sim_oracle as SO
from paper_2501_11779_amd import binding as G
from tests.test_abi_host import _emulate_balanced_split, good

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
NATIVE = os.path.join(ROOT, "tests", "native")
SAN = ["-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
       "-fno-sanitize-recover=all", "-static-libasan", "-static-libubsan"]
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=0:abort_on_error=0",
           UBSAN_OPTIONS="halt_on_error=1:print_stacktrace=1")


def build(tmp_path_factory, name, cmd):
    if shutil.which(cmd[0]) is None:
        pytest.skip(f"{cmd[0]} not available")
    exe = str(tmp_path_factory.mktemp("san") / name)
    res = subprocess.run([*cmd, "-o", exe], capture_output=True, text=True)
    assert res.returncode == 0, res.stderr
    return exe


def run(exe, args=(), stdin=None):
    res = subprocess.run([exe, *args], input=stdin, capture_output=True, text=True, env=ENV,
                         timeout=600)
    assert res.returncode == 0 and "runtime error" not in res.stderr and "Sanitizer" not in res.stderr, \
        f"{os.path.basename(exe)} failed ({res.returncode}):\n{res.stderr[-3000:]}"
    return res.stdout


@pytest.fixture(scope="module")
def oracle_exe(tmp_path_factory):
    return build(tmp_path_factory, "oracle_driver",
                 ["gcc", "-std=c11", *SAN, "-fopenmp", "-ffp-contract=off", "-Wall",
                  os.path.join(NATIVE, "oracle_driver.c"), "-lm"])


@pytest.fixture(scope="module")
def sim_exe(tmp_path_factory):
    return build(tmp_path_factory, "sim_driver",
                 ["g++", "-std=c++17", "-x", "c++", *SAN, "-Wall", "-I", os.path.join(ROOT, "include"),
                  os.path.join(NATIVE, "sim_driver.cpp")])


@pytest.fixture(scope="module")
def plan_exe(tmp_path_factory):
    return build(tmp_path_factory, "plan_driver",
                 ["g++", "-std=c++17", *SAN, "-Wall", "-I", os.path.join(ROOT, "include"),
                  os.path.join(NATIVE, "plan_driver.cpp")])


# ------------------------------------------------------------------ the oracle
def _layout(kind, n_slots, Hkv, cap, d, block_rows):
    if kind == "head_major":
        return (Hkv * cap * d, cap * d, d), (0, 0), n_slots * Hkv * cap * d
    if kind == "token_major":
        return (cap * Hkv * d, d, Hkv * d), (0, 0), n_slots * cap * Hkv * d
    assert cap % block_rows == 0
    return (cap * Hkv * d, block_rows * d, d), (block_rows, block_rows * Hkv * d), n_slots * cap * Hkv * d


@pytest.mark.parametrize("kind", ["head_major", "token_major", "head_blocked"])
@pytest.mark.parametrize("dtype", [O.F16, O.BF16])
def test_oracle_under_sanitizers_gives_the_same_bits(oracle_exe, tmp_path, kind, dtype):
    rng = np.random.default_rng(31 + dtype + len(kind))
    B, H, Hkv, d, cap, n_slots = 9, 6, 2, 128, 96, 11
    strides, block, cache_elems = _layout(kind, n_slots, Hkv, cap, d, 32)
    # lengths 0, 1, the last row of the slot; one slot id out of range, one position out of range
    pos = np.array([0, 1, cap - 1, 40, 17, 63, 5, cap, 30], dtype=np.int32)
    slot_id = rng.permutation(n_slots)[:B].astype(np.int32)
    slot_id[6] = n_slots + 3
    ctx_len = np.minimum(pos + 1, cap).astype(np.int32)

    def bits(shape):
        x = rng.standard_normal(shape).astype(np.float32)
        if dtype == O.F16:
            return x.astype(np.float16).view(np.uint16)
        return (x.view(np.uint32) >> 16).astype(np.uint16)

    q, k_new, v_new = bits((B, H, d)), bits((B, Hkv, d)), bits((B, Hkv, d))
    k_cache, v_cache = bits(cache_elems), bits(cache_elems)
    scale = float(np.float32(d ** -0.5))
    split_row = 33

    src = tmp_path / "problem.bin"
    with open(src, "wb") as f:
        f.write(struct.pack("<16q", B, H, Hkv, d, dtype, n_slots, cap, *strides, block[0], block[1],
                            cache_elems, split_row, 0, 0))
        f.write(struct.pack("<d", scale))
        for arr in (q, k_new, v_new, k_cache, v_cache, slot_id, pos, ctx_len):
            f.write(np.ascontiguousarray(arr).tobytes())
    dst = tmp_path / "result.bin"
    stdout = run(oracle_exe, [str(src), str(dst)])

    # the ordinary build on the same bytes
    p = O.make_problem(B, H, Hkv, d, dtype, n_slots, cap, scale, strides, block)
    kc, vc = k_cache.copy(), v_cache.copy()
    skipped = O.kv_append(p, kc, vc, k_new, v_new, slot_id, pos)
    want = O.decode_attention(p, q, kc, vc, slot_id, ctx_len)
    raw = open(dst, "rb").read()
    n = B * H * d
    assert struct.unpack_from("<i", raw, 0)[0] == skipped == 2
    got = np.frombuffer(raw, dtype=np.float64, count=n, offset=4).reshape(B, H, d)
    merged = np.frombuffer(raw, dtype=np.float64, count=n, offset=4 + 8 * n).reshape(B, H, d)
    tail = np.frombuffer(raw, dtype=np.uint16, offset=4 + 16 * n)
    assert np.array_equal(got.view(np.uint64), want.view(np.uint64))
    assert np.array_equal(tail[:cache_elems], kc) and np.array_equal(tail[cache_elems:], vc)
    # the split form merged again is the unsplit result (to float64 rounding)
    assert np.abs(merged - want).max() < 1e-12
    assert not want[6].any() and np.abs(want[0]).max() > 0
    # decoders: all 65 536 patterns went through; 2 * 1024 resp. 2 * 128 are inf or nan
    _, s16, odd16, sbf, oddbf = stdout.split()
    assert int(odd16) == 2048 and int(oddbf) == 256
    f16_sum = float(np.abs(np.arange(65536, dtype=np.uint16).view(np.float16)[
        np.isfinite(np.arange(65536, dtype=np.uint16).view(np.float16))].astype(np.float64)).sum())
    assert float.fromhex(s16) == pytest.approx(f16_sum, rel=1e-12)


# ------------------------------------------------------------------ the simulators
def test_simulators_under_sanitizers_match_the_python_oracle(sim_exe):
    rng = np.random.default_rng(2025)
    lines, wants = [], []
    for case in range(60):
        two = case % 2 == 0
        K = int(rng.choice([1, 2, 4]))
        N = K * int(rng.integers(1, 5))
        IF = int(rng.integers(1, 9))
        E = int(rng.integers(3, 7))
        later = int(rng.integers(0, 2))
        t = [float(x) for x in rng.uniform(0.05, 2.0, size=5).round(3)]
        if two:
            lines.append(f"two {N} {K} {IF} {E} {t[0]!r} {t[1]!r} {t[2]!r} {t[3]!r} {t[4]!r} {later}")
            wants.append(SO.two_tier(N, K, IF, E, t[0], t[1], t[2], t[3], t[4], later_first=bool(later)))
        else:
            lines.append(f"single {N} {K} {IF} {E} {t[0]!r} {t[1]!r} {t[2]!r} {later}")
            wants.append(SO.single_tier(N, K, IF, E, t[0], t[1], t[2], later_first=bool(later)))
    lines.append("two 8 3 2 4 0.1 0.1 0.1 0.1 0.1 0")             # N % K != 0: refused
    out = run(sim_exe, stdin="\n".join(lines) + "\n").strip().splitlines()
    assert len(out) == 61 and out[-1] == "-2"
    for line, want in zip(out, wants):
        fields = line.split()
        assert fields[0] == "0"
        got = [float.fromhex(x) for x in fields[1:]]
        assert got == list(want), (line, want)


# ------------------------------------------------------------------ the launch plan
def test_balanced_split_replayed_in_cpp_agrees_with_the_python_emulation(plan_exe):
    rng = np.random.default_rng(77)
    problems, lines = [], []
    for _ in range(120):
        T = int(rng.choice([1, 1, 1, 2, 4, 16, 64]))
        groups = int(rng.choice([1, 2, 3, 17, 64, 300, 1024, 4096]))
        Hkv = int(rng.choice([1, 2, 8]))
        G_ = int(rng.choice([1, 4, 8, 20, 40]))
        max_ctx = int(rng.choice([1, 31, 32, 33, 100, 1000, 4097, 32769]))
        if groups * T > 8192:
            groups = 8192 // T
        kind = rng.integers(0, 4)
        if kind == 0:
            rows = np.full(groups, max_ctx)
        elif kind == 1:
            rows = np.zeros(groups, dtype=np.int64)
            rows[rng.integers(0, groups)] = max_ctx
        elif kind == 2:
            rows = rng.integers(0, max_ctx + 1, size=groups)
        else:
            rows = np.where(rng.random(groups) < 0.9, rng.integers(0, 3, size=groups), max_ctx)
        rows = [int(r) for r in rows]
        problems.append((groups, T, Hkv, G_, max_ctx, rows))
        lines.append(f"{groups * T} {Hkv * G_} {Hkv} {max_ctx} {T} {groups} " + " ".join(map(str, rows)))
    out = run(plan_exe, stdin="\n".join(lines) + "\n").strip().splitlines()
    assert len(out) == len(problems)
    for line, (groups, T, Hkv, G_, max_ctx, rows) in zip(out, problems):
        assert line.startswith("PLAN "), line
        f = line.split()
        p = good(batch=groups * T, n_q_heads=Hkv * G_, n_kv_heads=Hkv, n_slots=groups,
                 slot_capacity=max_ctx, max_ctx_len=max_ctx,
                 strides=(Hkv * max_ctx * 128, max_ctx * 128, 128), tokens_per_group=T)
        plan = G.gh_decode_split_plan(p)
        assert [int(x) for x in f[1:7]] == [plan.n_workers, plan.min_share, plan.passes_per_strip,
                                            plan.waves_per_worker, plan.strips_per_kv_head,
                                            plan.n_chunks]
        pieces, _, _ = _emulate_balanced_split(plan, rows, Hkv)
        assert [int(x) for x in f[8:]] == [len(ps) for ps in pieces]
        assert max(len(ps) for ps in pieces) <= plan.n_chunks

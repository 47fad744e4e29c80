"""Shared plumbing of the parity tests: host copies for the oracle, tolerances."""
import numpy as np

from oracle import gh_oracle as O
from paper_2501_11779_amd import workloads as W

MAX_ABS_TOL = 2e-3      # spec tolerance for 16-bit K/V with fp32 accumulation
REL_L2_TOL = 1e-3


def errors(got, want):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    max_abs = float(np.abs(got - want).max()) if got.size else 0.0
    den = float(np.linalg.norm(want.ravel()))
    rel_l2 = float(np.linalg.norm((got - want).ravel()) / den) if den > 0 else 0.0
    return max_abs, rel_l2


def assert_parity(got, want, what=""):
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    max_abs, rel_l2 = errors(got, want)
    assert max_abs <= MAX_ABS_TOL and rel_l2 <= REL_L2_TOL, \
        f"{what}: max_abs={max_abs:.3e} rel_l2={rel_l2:.3e}"
    return max_abs, rel_l2


def host_copy(inp):
    """Bit patterns of every 16-bit tensor of a make_inputs() dict, before the step runs."""
    return {
        "q": W.bits(inp["q"]), "k_new": W.bits(inp["k_new"]), "v_new": W.bits(inp["v_new"]),
        "k_cache": W.bits(inp["k_cache"]), "v_cache": W.bits(inp["v_cache"]),
        "slot_id": inp["slot_id"].cpu().numpy().astype(np.int32),
        "pos": inp["pos"].cpu().numpy().astype(np.int32),
        "ctx_len": inp["ctx_len"].cpu().numpy().astype(np.int32),
    }


def oracle_problem(inp, batch=None, n_slots=None):
    w = inp["workload"]
    return O.make_problem(batch if batch is not None else w.batch, w.n_q_heads, w.n_kv_heads,
                          w.head_dim, W.DTYPE_CODE[w.dtype],
                          n_slots if n_slots is not None else inp["n_slots"], inp["capacity"],
                          inp["scale"], inp["strides"] if n_slots is None else
                          W.cache_shape_and_strides(n_slots, w.n_kv_heads, inp["capacity"],
                                                    w.head_dim, inp["layout"],
                                                    inp.get("block", (0, 0))[0])[1],
                          block=inp.get("block", (0, 0)))


def oracle_step(inp, host, append=True):
    """Oracle append (into the host mirror, in place) followed by oracle attention."""
    p = oracle_problem(inp)
    if append:
        skipped = O.kv_append(p, host["k_cache"], host["v_cache"], host["k_new"], host["v_new"],
                              host["slot_id"], host["pos"])
        assert skipped == 0
    return O.decode_attention(p, host["q"], host["k_cache"], host["v_cache"], host["slot_id"],
                              host["ctx_len"])


def sequence_slice(inp, b):
    """Host copy of one sequence as a batch-of-one problem on a one-slot cache (pre-step bits)."""
    slot = int(inp["slots"][b])
    return {
        "q": W.bits(inp["q"][b:b + 1]), "k_new": W.bits(inp["k_new"][b:b + 1]),
        "v_new": W.bits(inp["v_new"][b:b + 1]),
        "k_cache": W.bits(inp["k_cache"][slot:slot + 1]),
        "v_cache": W.bits(inp["v_cache"][slot:slot + 1]),
        "slot_id": np.zeros(1, dtype=np.int32),
        "pos": np.array([inp["lengths"][b]], dtype=np.int32),
        "ctx_len": np.array([inp["lengths"][b] + 1], dtype=np.int32),
    }


def oracle_sequence(inp, host1):
    """Oracle append + attention for a sequence_slice(); returns (out[H,d], k_mirror, v_mirror)."""
    p = oracle_problem(inp, batch=1, n_slots=1)
    assert O.kv_append(p, host1["k_cache"], host1["v_cache"], host1["k_new"], host1["v_new"],
                       host1["slot_id"], host1["pos"]) == 0
    out = O.decode_attention(p, host1["q"], host1["k_cache"], host1["v_cache"], host1["slot_id"],
                             host1["ctx_len"])
    return out[0], host1["k_cache"], host1["v_cache"]

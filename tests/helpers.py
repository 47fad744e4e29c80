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


# What the kernels actually deliver, with margin (measured worst case over the full-size workloads:
# max-abs 4.7e-6, rel-L2 2.4e-6): 16-bit products are exact in fp32, the sums are fp32, and the
# probabilities enter the P.V matrix product as hi + lo pairs of 16-bit values.  A kernel that
# rounds the probabilities to one 16-bit value (bf16: 2^-9 relative) lands an order of magnitude
# above these bounds on N(0,1) data.
TIGHT_MAX_ABS = 5e-5
TIGHT_REL_L2 = 2e-5


def assert_tight(got, want, what=""):
    max_abs, rel_l2 = errors(got, want)
    assert max_abs <= TIGHT_MAX_ABS and rel_l2 <= TIGHT_REL_L2, \
        f"{what}: max_abs={max_abs:.3e} rel_l2={rel_l2:.3e} (regression bound)"
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


def round_f64_to_bits(x, dtype):
    """Correctly rounded (nearest, ties to even) 16-bit patterns of float64 values, without going
    through float32: the two neighbours in the 16-bit format are compared in float64."""
    x = np.asarray(x, dtype=np.float64)
    if dtype == "f16":
        return x.astype(np.float16).view(np.uint16)
    f32 = x.astype(np.float32)
    trunc = (f32.view(np.uint32) & 0xffff0000).astype(np.uint32)       # toward zero, 8-bit mantissa
    lo = trunc.view(np.float32).astype(np.float64)
    hi = (trunc + np.uint32(0x10000)).view(np.float32).astype(np.float64)  # next away from zero
    # float32 rounding may have carried past hi's neighbour; restart from the value below |x|
    swap = np.abs(lo) > np.abs(x)
    trunc = np.where(swap, trunc - np.uint32(0x10000), trunc).astype(np.uint32)
    lo = trunc.view(np.float32).astype(np.float64)
    hi = (trunc + np.uint32(0x10000)).view(np.float32).astype(np.float64)
    dlo, dhi = np.abs(x - lo), np.abs(hi - x)
    even_lo = ((trunc >> 16) & 1) == 0
    pick_hi = (dhi < dlo) | ((dhi == dlo) & ~even_lo)
    bits = np.where(pick_hi, trunc + np.uint32(0x10000), trunc) >> 16
    return bits.astype(np.uint16)


def ulps_apart(a_bits, b_bits):
    """Distance in representable values between two arrays of same-sign-or-zero 16-bit patterns."""
    def key(u):
        u = u.astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7fff), u & 0x7fff)
    return np.abs(key(a_bits) - key(b_bits))


def assert_rounded_within(got_bits, want, dtype, eps, what=""):
    """A 16-bit result is right if it is the correct rounding of SOME value within eps of the
    oracle's float64 result, eps being the absolute error bound asserted on the fp32 result:
    rounding is monotonic, so got must lie between round(want - eps) and round(want + eps).
    (Counting representable values apart says the same for |x| >> eps and means nothing next to
    zero, where a 16-bit step is far smaller than eps.)  Returns the fraction of values that equal
    the oracle rounded once."""
    def key(u):
        u = u.astype(np.int32)
        return np.where(u & 0x8000, -(u & 0x7fff), u & 0x7fff)
    want = np.asarray(want, dtype=np.float64)
    lo, hi = key(round_f64_to_bits(want - eps, dtype)), key(round_f64_to_bits(want + eps, dtype))
    g = key(np.asarray(got_bits))
    bad = (g < lo) | (g > hi)
    assert not bad.any(), f"{what}: {int(bad.sum())} 16-bit values outside the rounding of want +- {eps}"
    return float((np.asarray(got_bits) == round_f64_to_bits(want, dtype)).mean())


def record_counts(ws, batch, n_q_heads):
    """int32 n[B*H] of a workspace tensor (records in use per head; -1 = finished by the attention
    kernel): the words before the arrival counters that end the workspace."""
    import torch
    rows = batch * n_q_heads
    return ws.view(torch.int32)[-2 * rows:-rows].cpu().numpy()

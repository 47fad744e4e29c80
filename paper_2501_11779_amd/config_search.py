"""Exhaustive search for the two-tier configuration (K, K', B) (Section 4.2, Appendix C).

A configuration is scored by simulating the pipeline with the C++ simulator of this library
(include/gh_sim.h): compute and link occupation times come from per-batch-size profiles with
linear interpolation between the profiled sizes (Appendix C), links follow the alpha-beta model,
and the number of in-flight batches is what the Tier-2 context memory holds with the paper's
oversubscription factor.  This module holds only that glue; it imports no torch.

What the paper feeds the simulator with and this repository cannot: measured Tier-1 (non-attention)
kernel profiles of the accelerators it studies.  `tier1_roofline_profile` is a stand-in built from
the paper's own resource count for the non-attention operations (Appendix A, Table 5 totals) and a
device's memory bandwidth and matrix throughput; the Tier-2 curve is measured with this library's
kernels on an MI355X (profile_tier2.py).
"""
import bisect
import json
import math
import os
from dataclasses import dataclass

from . import sim

HERE = os.path.dirname(os.path.abspath(__file__))


def profile_batch_sizes(max_batch=4096):
    """1, 2, 3, 4, 6, 8, 12, 16, ...: a factor of about sqrt(2) apart (Appendix C)."""
    out, p = [], 1
    while p <= max_batch:
        out.append(p)
        if p >= 2 and p + p // 2 <= max_batch:
            out.append(p + p // 2)
        p *= 2
    return sorted(set(out))


@dataclass
class Profile:
    """Duration of one layer's operation against batch size; linear in between (Appendix C)."""
    batch: list
    seconds: list

    def __call__(self, b):
        xs, ys = self.batch, self.seconds
        if b <= xs[0]:
            return ys[0] * b / xs[0] if b < xs[0] else ys[0]
        if b >= xs[-1]:
            return ys[-1] * b / xs[-1]          # beyond the sweep: proportional to the batch
        i = bisect.bisect_right(xs, b)
        x0, x1, y0, y1 = xs[i - 1], xs[i], ys[i - 1], ys[i]
        return y0 + (y1 - y0) * (b - x0) / (x1 - x0)

    @classmethod
    def load(cls, path):
        d = json.load(open(path))
        return cls(list(d["batch"]), list(d["seconds"]))


@dataclass
class Model:
    n_layers: int       # N
    d_model: int        # D
    d_kv: int           # D_kv
    d_hidden: int       # D_h
    seq_len: int        # S, the maximum sequence length contexts are sized for
    bytes_per_elem: int = 2

    @property
    def context_bytes_per_prompt(self):
        """M = 4 * N * S * D_kv bytes at 2-byte elements (Section 3.1)."""
        return 2 * self.bytes_per_elem * self.n_layers * self.seq_len * self.d_kv

    def tier1_to_tier2_bytes(self, batch):
        """Per layer: 2 * (2D + 2D_kv) bytes per token (Section 5.4.3)."""
        return self.bytes_per_elem * (2 * self.d_model + 2 * self.d_kv) * batch

    def tier2_to_tier1_bytes(self, batch):
        """Per layer: 2 * D bytes per token (Section 5.4.3)."""
        return self.bytes_per_elem * self.d_model * batch


LLAMA2_70B = Model(n_layers=80, d_model=8192, d_kv=1024, d_hidden=28672, seq_len=2048)


def tier1_roofline_profile(model, mem_bw, flops, batches=None):
    """Non-attention time of one layer from Table 5's totals: weights plus activations moved once
    at `mem_bw` bytes/s, 2 flops per multiply-accumulate at `flops` per second; the larger wins."""
    D, Dh, Dkv, e = model.d_model, model.d_hidden, model.d_kv, model.bytes_per_elem
    batches = batches or profile_batch_sizes()
    secs = []
    for B in batches:
        elems = D * (2 * D + 3 * Dh + 2 * Dkv) + B * (8 * D + 3 * Dh + 2 * Dkv)
        macs = B * D * (2 * D + 3 * Dh + 2 * Dkv)
        secs.append(max(elems * e / mem_bw, 2 * macs / flops))
    return Profile(list(batches), secs)


@dataclass
class Link:
    rtt: float          # seconds, minimum round-trip time between tiers
    bandwidth: float    # bytes per second
    alpha: float = 0.0  # fixed per-message cost of the alpha-beta model, seconds

    def transfer(self, nbytes):
        return self.alpha + nbytes / self.bandwidth


@dataclass
class Candidate:
    K: int
    K_prime: int
    B: int
    in_flight: int
    tbt: float
    tokens_per_s: float
    score: float


def in_flight_batches(model, K, tier2_context_bytes, B, oversubscription):
    """Batches of B*K' prompts whose contexts fit the K*K' Tier-2 nodes: each node keeps the
    contexts of B prompts per batch for the N/K layers of its Tier-1 node (Section 4.2)."""
    per_node_per_batch = B * model.context_bytes_per_prompt / K
    return int(oversubscription * tier2_context_bytes // per_node_per_batch)


def evaluate(model, K, K_prime, B, tier1, tier2, link, tier2_context_bytes, oversubscription=3.0,
             iterations=8, later_first=True):
    """Simulated tokens/s of one configuration (None if not even one batch fits)."""
    n_if = in_flight_batches(model, K, tier2_context_bytes, B, oversubscription)
    if n_if < 1:
        return None
    t1_batch = B * K_prime
    gen = sim.gh_sim_two_tier(
        model.n_layers, K, n_if, iterations,
        link.transfer(model.tier1_to_tier2_bytes(t1_batch)),
        link.transfer(model.tier2_to_tier1_bytes(t1_batch)),
        link.rtt, tier2(B), tier1(t1_batch), later_first)
    tbt = sim.gh_sim_tbt(gen, 2)
    return n_if, tbt, t1_batch * n_if / tbt


def search(model, tier1, tier2, link, tier2_context_bytes, max_tier1_nodes, max_tier2_per_tier1,
           batches=None, oversubscription=3.0, cost=None, max_in_flight=512):
    """argmax over (K, K', B) of tokens/s, or of tokens/s per cost when `cost(K, K')` is given.
    K runs over the divisors of N (every node hosts the same number of layers).  Returns the
    candidates sorted best first."""
    batches = batches or profile_batch_sizes()
    out = []
    for K in range(1, max_tier1_nodes + 1):
        if model.n_layers % K:
            continue
        for Kp in range(1, max_tier2_per_tier1 + 1):
            for B in batches:
                n_if = in_flight_batches(model, K, tier2_context_bytes, B, oversubscription)
                if n_if < 1 or n_if > max_in_flight:
                    continue
                r = evaluate(model, K, Kp, B, tier1, tier2, link, tier2_context_bytes, oversubscription)
                if r is None:
                    continue
                n_if, tbt, tps = r
                score = tps / cost(K, Kp) if cost else tps
                out.append(Candidate(K, Kp, B, n_if, tbt, tps, score))
    out.sort(key=lambda c: -c.score)
    return out


def measured_tier2_profile(name="tier2_mi355x_llama2_70b.json"):
    """The Tier-2 curve measured on an MI355X with this library (written by profile_tier2.py)."""
    return Profile.load(os.path.join(HERE, "data", name))


def main():
    """Worked example: Llama2-70B, Tier 1 from the roofline stand-in, Tier 2 from the measured
    MI355X curve.  `python -m paper_2501_11779_amd.config_search`"""
    import argparse
    import time
    ap = argparse.ArgumentParser()
    ap.add_argument("--tier1-bandwidth", type=float, default=6.4e12, help="bytes/s (default 80%% of 8 TB/s)")
    ap.add_argument("--tier1-flops", type=float, default=1.5e15, help="flop/s reached by the Tier-1 GEMMs")
    ap.add_argument("--link-bandwidth", type=float, default=50e9, help="bytes/s between the tiers")
    ap.add_argument("--link-rtt", type=float, default=20e-6, help="seconds")
    ap.add_argument("--tier2-context-gib", type=float, default=200.0, help="context memory per Tier-2 device")
    ap.add_argument("--max-tier1", type=int, default=8)
    ap.add_argument("--max-tier2-per-tier1", type=int, default=4)
    ap.add_argument("--top", type=int, default=5)
    args = ap.parse_args()
    tier2 = measured_tier2_profile()
    tier1 = tier1_roofline_profile(LLAMA2_70B, args.tier1_bandwidth, args.tier1_flops)
    link = Link(rtt=args.link_rtt, bandwidth=args.link_bandwidth)
    t0 = time.perf_counter()
    cands = search(LLAMA2_70B, tier1, tier2, link, args.tier2_context_gib * 2 ** 30, args.max_tier1,
                   args.max_tier2_per_tier1)
    print(f"{len(cands)} configurations simulated in {time.perf_counter() - t0:.1f} s")
    for c in cands[:args.top]:
        print(f"K={c.K} K'={c.K_prime} B={c.B} in-flight={c.in_flight} TBT={c.tbt * 1e3:.1f} ms "
              f"{c.tokens_per_s:.3e} tokens/s")


if __name__ == "__main__":
    main()

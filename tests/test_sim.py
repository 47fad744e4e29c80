"""Pipeline simulators and in-flight-batch calculus: the plain-Python oracle against closed forms
and the paper's worked examples, then the C++ simulator against the oracle (no GPU needed)."""
import os
import random

import pytest

from oracle import sim_oracle as SO
from paper_2501_11779_amd import sim as S

HERE = os.path.dirname(os.path.abspath(__file__))


def _examples():
    rows = []
    for ln in open(os.path.join(HERE, "golden", "in_flight_examples.txt")):
        if ln.strip() and not ln.startswith("#"):
            f = ln.split()
            rows.append((f[0], int(f[1]), int(f[2]), float(f[3]), float(f[4]), int(f[5]), int(f[6]), int(f[7])))
    return rows


# ------------------------------------------------------------------ closed forms (oracle)
@pytest.mark.parametrize("scheme,K,N,t_n,t_c,IF,fit,max_b", _examples())
def test_paper_worked_examples(scheme, K, N, t_n, t_c, IF, fit, max_b):
    for mod in (SO, None):
        if scheme == "pp":
            got = SO.if_pp(K, N, t_n, t_c) if mod else S.gh_sim_if_pp(K, N, t_n, t_c)
        else:
            got = SO.if_tp(K, t_n, t_c) if mod else S.gh_sim_if_tp(K, t_n, t_c)
        assert got == IF
        assert (SO.max_batch(fit, 1, IF) if mod else S.gh_sim_max_batch(fit, 1, IF)) == max_b


def test_eq2_two_tier_in_flight():
    assert SO.if_gh(0.8, 2.2, 1.0) == 4 == S.gh_sim_if_gh(0.8, 2.2, 1.0)
    assert SO.if_gh(0.0, 0.0, 1.0) == 1 == S.gh_sim_if_gh(0.0, 0.0, 1.0)


def test_one_batch_sees_the_sum_of_all_latencies():
    """A single in-flight batch never queues: a token takes N times the six (three) stage latencies."""
    g = SO.two_tier(N=8, K=2, IF=1, E=6, t_net_12=0.3, t_net_21=0.2, t_net_rtt=1.0, t_c_att=0.7,
                    t_c_nonatt=1.1)
    per_layer = 1.1 + 0.3 + 0.5 + 0.7 + 0.2 + 0.5
    for a, b in zip(g, g[1:]):
        assert b - a == pytest.approx(8 * per_layer, rel=1e-12)
    g = SO.single_tier(N=6, K=3, IF=1, E=5, t_net_link=0.25, t_net_rtt=2.0, t_c=1.5)
    for a, b in zip(g, g[1:]):
        assert b - a == pytest.approx(6 * (1.5 + 0.25 + 1.0), rel=1e-12)


def _settled_gap(g):
    """Mean token spacing over the second half of the run (batch 0's own spacing jitters a little
    around the pipeline's period)."""
    half = len(g) // 2
    return (g[-1] - g[half]) / (len(g) - 1 - half)


def test_many_batches_are_bound_by_the_busiest_queue():
    """With plenty of batches in flight and later stages served first, the slowest single-consumer
    pipe is always busy: each of the IF batches occupies it N/K times per pass, so
    TBT = IF * (N/K) * max(queue latencies)."""
    N, K, IF = 8, 2, 40
    g = SO.two_tier(N, K, IF, 40, t_net_12=0.3, t_net_21=0.2, t_net_rtt=1.0, t_c_att=0.7, t_c_nonatt=1.1)
    assert _settled_gap(g) == pytest.approx(IF * (N // K) * 1.1, rel=2e-3)
    g = SO.two_tier(N, K, IF, 40, t_net_12=0.3, t_net_21=0.2, t_net_rtt=1.0, t_c_att=1.9, t_c_nonatt=1.1)
    assert _settled_gap(g) == pytest.approx(IF * (N // K) * 1.9, rel=2e-3)      # Tier 2 too slow
    g = SO.single_tier(N, K, IF, 40, t_net_link=2.5, t_net_rtt=0.5, t_c=1.0)
    assert _settled_gap(g) == pytest.approx(IF * (N // K) * 2.5, rel=2e-3)      # link-bound
    # one node: nothing to pipeline, both service orders give the bound exactly
    for later in (False, True):
        g = SO.two_tier(N, 1, IF, 30, 0.3, 0.2, 1.0, 0.7, 1.1, later_first=later)
        assert _settled_gap(g) == pytest.approx(IF * N * 1.1, rel=2e-3)


def test_listing_order_leaves_pipeline_stages_idle():
    """Serving the earliest stage first (the listing as printed) keeps the batches in one clump:
    a K = 2 pipeline then needs clearly more than the busiest queue's time per token."""
    N, K, IF = 8, 2, 40
    clump = SO.tbt(SO.two_tier(N, K, IF, 10, 0.3, 0.2, 1.0, 0.7, 1.1, later_first=False))
    assert clump > 1.4 * IF * (N // K) * 1.1


def test_throughput_saturates_at_the_in_flight_count_of_eq2():
    """One Tier-1 node: tokens per time grow with IF until the Tier-2 round trip is hidden, which
    is Eq. 2's count, and stay flat afterwards."""
    N, B = 4, 16
    t_att, t_12, t_21, rtt, t_non = 0.8, 0.1, 0.1, 2.0, 1.0
    knee = SO.if_gh(t_att, t_12 + t_21 + rtt, t_non)
    assert knee == 4
    rates = []
    for IF in range(1, 9):
        g = SO.two_tier(N, 1, IF, 8, t_12, t_21, rtt, t_att, t_non)
        rates.append(SO.throughput(B, IF, g))
    for IF in range(1, knee):
        assert rates[IF] > rates[IF - 1] * 1.2          # still growing below the knee
    for IF in range(knee, 8):
        assert rates[IF] == pytest.approx(B / t_non / N * 1.0 * N / N, rel=1e-9) or \
            rates[IF] == pytest.approx(rates[knee - 1], rel=1e-9)
    assert rates[knee - 1] == pytest.approx(B * knee / (knee * N * t_non), rel=1e-9)


def test_pipeline_parallel_needs_eq1_batches():
    """K single-tier stages, one block of layers per node (the listing charges the link after
    every simulated layer, so a node's layers are one simulated layer here), with a transfer half
    as long as the stage compute: K batches leave every node idle a third of the time, Eq. 1's 2K
    batches keep them busy."""
    K = N = 4
    t_c, t_link, rtt = 2.0, 0.5, 1.0               # t_n = link + rtt/2 = 1 <= t_c
    need = SO.if_pp(K, N, t_link + rtt / 2, t_c)
    assert need == 2 * K
    full = _settled_gap(SO.single_tier(N, K, need, 40, t_link, rtt, t_c)) / need
    half = _settled_gap(SO.single_tier(N, K, K, 40, t_link, rtt, t_c)) / K
    assert full == pytest.approx(t_c, rel=2e-3)                  # compute-bound: no idle time
    assert half == pytest.approx(t_c + t_link + rtt / 2, rel=2e-3)


# ------------------------------------------------------------------ product against oracle
def test_cpp_simulator_matches_oracle_exactly():
    rng = random.Random(7)
    for trial in range(60):
        K = rng.choice([1, 2, 3, 4])
        N = K * rng.choice([1, 2, 3, 5])
        IF = rng.randint(1, 14)
        E = rng.randint(3, 7)
        later = rng.random() < 0.5
        t = [rng.choice([0.0, 0.1, 0.25, 0.5, 1.0, 1.7, 3.0]) for _ in range(5)]
        if trial % 2 == 0:
            want = SO.two_tier(N, K, IF, E, t[0], t[1], t[2], t[3], t[4] + 0.1, later)
            got = S.gh_sim_two_tier(N, K, IF, E, t[0], t[1], t[2], t[3], t[4] + 0.1, later)
        else:
            want = SO.single_tier(N, K, IF, E, t[0], t[1], t[2] + 0.1, later)
            got = S.gh_sim_single_tier(N, K, IF, E, t[0], t[1], t[2] + 0.1, later)
        assert got == want, (trial, N, K, IF, E, later, t)
        assert S.gh_sim_tbt(got, 1) == pytest.approx(SO.tbt(want, 1), rel=1e-15) if E >= 3 else True


def test_cpp_simulator_argument_checks():
    L = S.lib()
    import ctypes as C
    out = (C.c_double * 4)()
    assert L.gh_sim_two_tier(8, 3, 2, 4, 0.1, 0.1, 0.1, 0.1, 0.1, 0, out) == -2     # N % K != 0
    assert L.gh_sim_two_tier(8, 2, 0, 4, 0.1, 0.1, 0.1, 0.1, 0.1, 0, out) == -2
    assert L.gh_sim_single_tier(8, 2, 2, 4, 0.1, 0.1, 0.1, 0, None) == -1
    assert L.gh_sim_tbt(out, 3, 2) < 0
    assert S.gh_sim_max_batch(32.0, 0.0, 4) == 0


def test_sim_symbols_exported():
    import re
    text = open(os.path.join(os.path.dirname(HERE), "include", "gh_sim.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(gh_sim_[a-z_0-9]+)\s*\(", text))
    assert names == set(S.SIM_EXPORTS)
    for n in names:
        assert getattr(S.lib(), n) is not None


# ------------------------------------------------------------------ configuration search
def test_profile_grid_and_interpolation():
    from paper_2501_11779_amd import config_search as CS
    grid = CS.profile_batch_sizes(64)
    assert grid == [1, 2, 3, 4, 6, 8, 12, 16, 24, 32, 48, 64]          # Appendix C's example grid
    p = CS.Profile([4, 6, 8], [1.0, 2.0, 2.5])
    assert p(5) == pytest.approx(1.5)                                   # "average of 4 and 6"
    assert p(4) == 1.0 and p(8) == 2.5 and p(7) == pytest.approx(2.25)
    assert p(16) == pytest.approx(5.0) and p(2) == pytest.approx(0.5)   # outside: proportional


def test_context_memory_and_message_sizes_follow_the_paper():
    from paper_2501_11779_amd import config_search as CS
    m = CS.LLAMA2_70B
    assert m.context_bytes_per_prompt == 640 * 2 ** 20                  # Section 3.1's example
    assert m.tier1_to_tier2_bytes(1) == 2 * (2 * 8192 + 2 * 1024)      # Section 5.4.3
    assert m.tier2_to_tier1_bytes(3) == 3 * 2 * 8192
    # 10 Tier-1 nodes, 64 GiB of context per Tier-2 node, 3x oversubscription, B = 96
    assert CS.in_flight_batches(m, 10, 64 * 2 ** 30, 96, 3.0) == int(3 * 64 * 2 ** 30 // (96 * 64 * 2 ** 20))


def test_search_agrees_with_brute_force_over_the_oracle_simulator():
    from paper_2501_11779_amd import config_search as CS
    m = CS.Model(n_layers=8, d_model=256, d_kv=64, d_hidden=512, seq_len=128)
    tier1 = CS.Profile([1, 64, 4096], [1e-4, 1.2e-4, 4e-3])
    tier2 = CS.Profile([1, 16, 4096], [2e-5, 6e-5, 1.2e-2])
    link = CS.Link(rtt=2e-4, bandwidth=1e9)
    ctx = 6 * 2 ** 20
    cands = CS.search(m, tier1, tier2, link, ctx, max_tier1_nodes=4, max_tier2_per_tier1=3,
                      batches=[1, 2, 4, 8, 16], oversubscription=3.0)
    assert cands and cands[0].score == max(c.score for c in cands)
    best = None
    for K in (1, 2, 4):
        for Kp in (1, 2, 3):
            for B in (1, 2, 4, 8, 16):
                n_if = int(3.0 * ctx // (B * m.context_bytes_per_prompt / K))
                if n_if < 1:
                    continue
                g = SO.two_tier(m.n_layers, K, n_if, 8, link.transfer(m.tier1_to_tier2_bytes(B * Kp)),
                                link.transfer(m.tier2_to_tier1_bytes(B * Kp)), link.rtt, tier2(B),
                                tier1(B * Kp))
                tps = SO.throughput(B * Kp, n_if, g)
                if best is None or tps > best[0]:
                    best = (tps, K, Kp, B)
    assert (cands[0].K, cands[0].K_prime, cands[0].B) == best[1:]
    assert cands[0].tokens_per_s == pytest.approx(best[0], rel=1e-12)


def test_measured_tier2_curve_is_loadable_and_sane():
    from paper_2501_11779_amd import config_search as CS
    p = CS.measured_tier2_profile()
    assert p.batch == CS.profile_batch_sizes(4096)
    assert all(b > a for a, b in zip(p.seconds, p.seconds[1:]))          # more work takes longer
    assert 1e5 < 1024 / p(1024) < 2e6                                    # sequence-steps/s

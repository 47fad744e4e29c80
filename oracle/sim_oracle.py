"""Plain-Python reference of the paper's pipeline simulations and in-flight-batch calculus.

TEST INFRASTRUCTURE ONLY (like the rest of oracle/): slow, written step by step in the paper's
order and notation, imported by tests only.  It shares no code with the C++ simulator of the
product library.

What it follows:
  * Appendix C, Algorithm 1 (two-tier simulation): every layer has six stages -- Tier-1
    non-attention compute, Tier-1 -> Tier-2 link, half the inter-tier RTT, Tier-2 attention,
    Tier-2 -> Tier-1 link, half the RTT.  6K pipes (one set of six per Tier-1 node), each a
    single-consumer queue except the RTT pipes, which are pure delays.  IF batches start in pipe 0;
    the loop always serves the pipe with the nearest event, pops from it -- among the events that
    have arrived by then -- the one with the earliest stage, then the earliest timestamp, occupies
    the pipe for the stage's latency and forwards the event to the pipe of its next stage.  The
    times at which batch 0 wraps around to stage 0 are returned.
  * Appendix C, Algorithm 2 (single-tier simulation): the same with three stages per layer
    (compute, node-to-node link, half the RTT) and 3K pipes.
  * Section 3.2, Eq. 1 (pipeline parallelism), Section 3.3, Eq. 2 (two tiers), Appendix B, Eq. 3
    (tensor parallelism): in-flight batches needed for full utilisation; Section 3.1: the largest
    batch is floor(C_max / (M * IF)).
  * Appendix C, closing paragraph: TBT is the spacing of batch 0's arrivals at the first layer
    after two warm-up passes, throughput = B * IF / TBT.

Readings where the listing is silent or at odds with the prose:
  * "pop(.timestamp < next_event_ts[w])" is read as "<=": when a pipe is idle its next event time
    IS the timestamp of its earliest event, which must be eligible.
  * stage_to_pipes: layer l lives on Tier-1 node l // (N / K) (N divisible by K), stage s of that
    layer uses that node's pipe number s mod 6 (or mod 3).
  * Ties: argmin picks the lowest pipe index; equal (stage, timestamp) pops the lowest batch id.
  * The listing pops the EARLIEST stage first, while Section 4.1.1 and the prose of Appendix C say
    that batches further along are served first.  Both are implemented.  With the listing's order
    the in-flight batches travel as one clump and the Tier-1 nodes of a K > 1 pipeline take turns
    idling (tests/test_sim.py shows it); with the prose's order the busiest queue stays busy, which
    is what the paper's throughput argument assumes.  later_first=True (the prose) is the default.
  * The listing logs `timestamp` (when the event entered its last stage), not the finish time;
    TBT is a difference, so the constant offset does not matter.  Followed as printed.
  * Eq. 1 is printed as ceil(1 + K*t_n / (N*t_c)) * K in Section 3.2 and with N and K swapped in
    Table 3; the prose (t_n against the compute of N/K layers) supports Section 3.2's form.
"""
import math

INF = float("inf")


def _simulate(larr, N, K, IF, E, later_first=True):
    S = len(larr)                      # stages per layer: 6 (two tiers) or 3 (single tier)
    assert N % K == 0 and IF >= 1 and E >= 1
    n_pipes = S * K
    pipes = [[] for _ in range(n_pipes)]          # lists of (stage, timestamp, id)
    layers_per_node = N // K

    def stage_to_pipe(stage):
        layer = stage // S
        return (layer // layers_per_node) * S + stage % S

    busy_till_ts = [0.0] * n_pipes
    next_event_ts = [INF] * n_pipes
    gen_ts = []

    def earliest(pipe):
        return min(ev[1] for ev in pipe) if pipe else INF

    for i in range(IF):
        pipes[0].append((0, 0.0, i))
    next_event_ts[0] = 0.0
    while len(gen_ts) < E:
        w = min(range(n_pipes), key=lambda i: next_event_ts[i])
        assert next_event_ts[w] < INF, "no event left"
        arrived = [ev for ev in pipes[w] if ev[1] <= next_event_ts[w]]
        if later_first:
            ev = min(arrived, key=lambda e: (-e[0], e[1], e[2]))
        else:
            ev = min(arrived, key=lambda e: (e[0], e[1], e[2]))
        pipes[w].remove(ev)
        stage, timestamp, bid = ev
        next_event_ts[w] = max(busy_till_ts[w], earliest(pipes[w]))

        delay = larr[stage % S]
        if stage % 3 != 2:
            finish_ts = max(busy_till_ts[w], timestamp) + delay
            busy_till_ts[w] = finish_ts
        else:
            finish_ts = timestamp + delay
        stage = (stage + 1) % (S * N)
        nw = stage_to_pipe(stage)
        pipes[nw].append((stage, finish_ts, bid))
        next_event_ts[nw] = max(busy_till_ts[nw], earliest(pipes[nw]))
        if stage == 0 and bid == 0:
            gen_ts.append(timestamp)
    return gen_ts


def two_tier(N, K, IF, E, t_net_12, t_net_21, t_net_rtt, t_c_att, t_c_nonatt, later_first=True):
    """Algorithm 1.  Returns the token generation times of batch 0."""
    larr = [t_c_nonatt, t_net_12, t_net_rtt / 2, t_c_att, t_net_21, t_net_rtt / 2]
    return _simulate(larr, N, K, IF, E, later_first)


def single_tier(N, K, IF, E, t_net_link, t_net_rtt, t_c, later_first=True):
    """Algorithm 2.  Returns the token generation times of batch 0."""
    larr = [t_c, t_net_link, t_net_rtt / 2]
    return _simulate(larr, N, K, IF, E, later_first)


def tbt(gen_ts, warmup=2):
    """Time between tokens once the pipeline has settled (two passes are discarded)."""
    assert len(gen_ts) >= warmup + 2
    return (gen_ts[-1] - gen_ts[warmup]) / (len(gen_ts) - 1 - warmup)


def throughput(B, IF, gen_ts, warmup=2):
    """Tokens per unit time: B * IF tokens per pass."""
    return B * IF / tbt(gen_ts, warmup)


def if_pp(K, N, t_n, t_c):
    """Eq. 1: in-flight batches that keep K pipeline stages busy."""
    return math.ceil(1 + K * t_n / (N * t_c)) * K


def if_gh(t_c2_att, t_n, t_c1_noatt):
    """Eq. 2: in-flight batches that hide the Tier-2 round trip from a Tier-1 node."""
    return math.ceil(1 + (t_c2_att + t_n) / t_c1_noatt)


def if_tp(K, t_n, t_c_min):
    """Eq. 3: in-flight batches for asynchronous K-way tensor parallelism."""
    return math.ceil(1 + t_n / (t_c_min / K))


def max_batch(C_max, M, n_in_flight):
    """Largest batch whose in-flight copies fit the context memory (Section 3.1 / 3.2)."""
    return int(C_max // (M * n_in_flight))

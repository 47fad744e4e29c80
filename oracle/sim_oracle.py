"""Plain-Python reference of the paper's pipeline simulations and in-flight-batch calculus.

TEST INFRASTRUCTURE ONLY (like the rest of oracle/): slow, a direct model of what Appendix C
describes -- stations that serve one batch at a time, delays, and the rule for choosing the next
batch -- imported by tests only.  It shares no code with the C++ simulator of the product library.

What it follows:
  * Appendix C, Algorithm 1 (two-tier simulation): every layer has six stages -- Tier-1
    non-attention compute, Tier-1 -> Tier-2 link, half the inter-tier RTT, Tier-2 attention,
    Tier-2 -> Tier-1 link, half the RTT.  6K stations (one set of six per Tier-1 node), each
    serving one batch at a time except the RTT stages, which are pure delays.  IF batches start at
    the first station; the station whose choice is due first chooses, among the batches that have
    arrived by then, by stage, then arrival time, then batch id, holds the batch for the stage's
    latency and passes it on.  The times at which batch 0 comes round to the first stage again are
    returned.
  * Appendix C, Algorithm 2 (single-tier simulation): the same with three stages per layer
    (compute, node-to-node link, half the RTT) and 3K stations.
  * Section 3.2, Eq. 1 (pipeline parallelism), Section 3.3, Eq. 2 (two tiers), Appendix B, Eq. 3
    (tensor parallelism): in-flight batches needed for full utilisation; Section 3.1: the largest
    batch is floor(C_max / (M * IF)).
  * Appendix C, closing paragraph: TBT is the spacing of batch 0's arrivals at the first layer
    after two warm-up passes, throughput = B * IF / TBT.

Readings where the listing is silent or at odds with the prose:
  * A batch counts as arrived when its arrival time is at or before the station's decision time
    (the listing writes a strict comparison; an idle station's decision time IS the arrival time
    of its earliest batch, which must be eligible).
  * Layer l lives on Tier-1 node l // (N / K) (N divisible by K); stage s of that layer uses that
    node's station number s mod 6 (or mod 3).
  * Ties: the first station in (node, stage) order chooses first; equal (stage, arrival) takes the
    lowest batch id.
  * When a station has chosen a batch, its next decision is scheduled from its state before that
    batch occupies it (the order of the listing's updates), so batches that are already waiting are
    committed behind it at once; see Station.choose.
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

NEVER = float("inf")


class Station:
    """One resource of the pipeline: a compute node, a link (one job at a time) or half a round
    trip (a pure delay: any number of jobs at once, nothing queues).  Jobs wait here as
    (hop, arrival time, batch) triples, `hop` counting the stages a batch has gone through since
    the first layer."""

    def __init__(self, latency, one_at_a_time):
        self.latency = latency
        self.one_at_a_time = one_at_a_time
        self.waiting = []
        self.free_at = 0.0          # when the job in service leaves (stays 0 for a delay)
        self.decide_at = NEVER      # when the station next chooses a job; NEVER: nothing waits

    def first_arrival(self):
        return min(job[1] for job in self.waiting) if self.waiting else NEVER

    def accept(self, job):
        """A job arrives: the choice is due once the station is free and something has arrived."""
        self.waiting.append(job)
        self.decide_at = max(self.free_at, self.first_arrival())

    def choose(self, further_along_first):
        """Takes, among the jobs that have arrived by the decision time, the one furthest along
        (or least far, with the listing's order), then the earliest arrival, then the lowest
        batch.  The next choice is scheduled from the station's state BEFORE this job occupies it
        (Appendix C's listing updates the pipe's next event before it marks the pipe busy): jobs
        that are already waiting are committed right behind this one, in priority order among
        themselves, and a job that arrives while they queue does not overtake them."""
        here = [job for job in self.waiting if job[1] <= self.decide_at]
        order = (lambda j: (-j[0], j[1], j[2])) if further_along_first else (lambda j: (j[0], j[1], j[2]))
        job = min(here, key=order)
        self.waiting.remove(job)
        self.decide_at = max(self.free_at, self.first_arrival())
        return job

    def serve(self, arrival):
        """Departure time of a job that arrived at `arrival`."""
        if not self.one_at_a_time:
            return arrival + self.latency
        self.free_at = max(self.free_at, arrival) + self.latency
        return self.free_at


def _simulate(stage_kinds, N, K, IF, E, later_first=True):
    """stage_kinds: (latency, one_at_a_time) of the stages of one layer, in order.  Every Tier-1
    node (N / K consecutive layers) owns one station per stage kind.  Returns E times at which
    batch 0 entered the last stage of a pass over all N layers."""
    per_layer = len(stage_kinds)
    assert N % K == 0 and IF >= 1 and E >= 1
    layers_per_node = N // K
    stations = [Station(lat, serial) for _ in range(K) for lat, serial in stage_kinds]
    hops_per_pass = per_layer * N

    def station_of(hop):
        node = (hop // per_layer) // layers_per_node
        return stations[node * per_layer + hop % per_layer]

    for batch in range(IF):
        stations[0].accept((0, 0.0, batch))
    passes = []
    while len(passes) < E:
        st = min(stations, key=lambda s: s.decide_at)        # nearest choice; first station on ties
        assert st.decide_at < NEVER, "no event left"
        hop, arrival, batch = st.choose(later_first)
        leaves = st.serve(arrival)
        hop = (hop + 1) % hops_per_pass
        station_of(hop).accept((hop, leaves, batch))
        if hop == 0 and batch == 0:
            passes.append(arrival)
    return passes


def two_tier(N, K, IF, E, t_net_12, t_net_21, t_net_rtt, t_c_att, t_c_nonatt, later_first=True):
    """Algorithm 1.  Returns the token generation times of batch 0."""
    layer = [(t_c_nonatt, True), (t_net_12, True), (t_net_rtt / 2, False),
             (t_c_att, True), (t_net_21, True), (t_net_rtt / 2, False)]
    return _simulate(layer, N, K, IF, E, later_first)


def single_tier(N, K, IF, E, t_net_link, t_net_rtt, t_c, later_first=True):
    """Algorithm 2.  Returns the token generation times of batch 0."""
    layer = [(t_c, True), (t_net_link, True), (t_net_rtt / 2, False)]
    return _simulate(layer, N, K, IF, E, later_first)


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

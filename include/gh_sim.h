/*
 * gh_sim.h -- the paper's pipeline simulations and in-flight-batch calculus
 * (host-only C ABI; no GPU involved).
 *
 * Appendix C models an inference pipeline as single-consumer queues (compute
 * nodes, links) and pure delays (half the round-trip time), sends IF in-flight
 * batches through it and reads the time between tokens of batch 0.  Algorithm 1
 * is the two-tier pipeline (six stages per layer: Tier-1 non-attention compute,
 * Tier-1 -> Tier-2 link, RTT/2, Tier-2 attention, Tier-2 -> Tier-1 link,
 * RTT/2), Algorithm 2 the single-tier pipeline (three stages per layer:
 * compute, link, RTT/2).  Layer l lives on Tier-1 node l / (N / K); each node
 * owns one pipe per stage kind.  The simulator always serves the pipe with the
 * nearest event (lowest index on ties), pops -- among the events that have
 * arrived by that time -- the earliest stage, then the earliest timestamp, then
 * the lowest batch id (later_first != 0 serves the latest stage first instead,
 * the rule the prose of Section 4.1.1 and Appendix C describes; with the
 * listing's order the batches of a K > 1 pipeline travel as one clump and the
 * nodes take turns idling, so callers normally pass 1), occupies the pipe for
 * the stage's latency and forwards the event.  A pipe's next choice is
 * scheduled from its state before the chosen batch occupies it (the order of
 * the updates in the printed algorithms): batches that were already waiting
 * are committed behind the chosen one at once, in priority order among
 * themselves, and a batch that arrives while they queue does not overtake them.
 *
 * All times are doubles in the caller's unit.  N must be divisible by K.
 * gen_ts receives E values: the times at which batch 0 wrapped around to the
 * first stage (as printed in the algorithms: the time it entered its last
 * stage).  Return: 0, -1 (null pointer), -2 (bad sizes).
 */
#ifndef GH_SIM_H
#define GH_SIM_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Algorithm 1. */
int32_t gh_sim_two_tier(int32_t N, int32_t K, int32_t IF, int32_t E, double t_net_12,
                        double t_net_21, double t_net_rtt, double t_c_att, double t_c_nonatt,
                        int32_t later_first, double* gen_ts);

/* Algorithm 2. */
int32_t gh_sim_single_tier(int32_t N, int32_t K, int32_t IF, int32_t E, double t_net_link,
                           double t_net_rtt, double t_c, int32_t later_first, double* gen_ts);

/* Time between tokens after `warmup` passes (Appendix C discards two): the mean spacing of
 * gen_ts[warmup .. E-1].  Needs E >= warmup + 2, else returns a negative value. */
double gh_sim_tbt(const double* gen_ts, int32_t E, int32_t warmup);

/* In-flight batches for full utilisation: Section 3.2 Eq. 1 (pipeline parallelism),
 * Section 3.3 Eq. 2 (two tiers), Appendix B Eq. 3 (tensor parallelism); and the largest batch
 * floor(C_max / (M * n_in_flight)) of Section 3.1. */
int32_t gh_sim_if_pp(int32_t K, int32_t N, double t_n, double t_c);
int32_t gh_sim_if_gh(double t_c2_att, double t_n, double t_c1_noatt);
int32_t gh_sim_if_tp(int32_t K, double t_n, double t_c_min);
int64_t gh_sim_max_batch(double C_max, double M, int32_t n_in_flight);

#ifdef __cplusplus
}
#endif
#endif /* GH_SIM_H */

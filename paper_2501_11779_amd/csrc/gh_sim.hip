// Discrete-event simulation of the single-tier and two-tier pipelines (host code only).
// Contract and the passages followed: include/gh_sim.h.
//
// Data structures differ from a literal reading of the algorithms (which scan every pipe and every
// queued event at each step): each pipe keeps its queue ordered by arrival time, so that only the
// events that have already arrived are looked at when choosing what to serve, and the pipes' next
// event times sit in one ordered set instead of being scanned.
#include "gh_sim.h"

#include <cmath>
#include <limits>
#include <set>
#include <tuple>
#include <vector>

namespace {

constexpr double kInf = std::numeric_limits<double>::infinity();

struct Event {
  int32_t stage;
  double ts;
  int32_t id;
};

struct Pipe {
  // (timestamp, stage, id): everything queued, for "earliest timestamp"
  std::set<std::tuple<double, int32_t, int32_t>> by_time;
  double busy_till = 0.0;
  double next_event = kInf;
};

int32_t simulate(const double* larr, int S, int32_t N, int32_t K, int32_t IF, int32_t E,
                 bool later_first, double* gen_ts) {
  if (!gen_ts) return -1;
  if (N <= 0 || K <= 0 || IF <= 0 || E <= 0 || N % K != 0) return -2;
  const int n_pipes = S * K;
  const int layers_per_node = N / K;
  std::vector<Pipe> pipes(n_pipes);
  std::set<std::pair<double, int>> agenda;          // (next event time, pipe) for finite times
  auto stage_to_pipe = [&](int32_t stage) {
    const int layer = stage / S;
    return (layer / layers_per_node) * S + stage % S;
  };
  auto set_next = [&](int w, double t) {
    Pipe& p = pipes[w];
    if (p.next_event != kInf) agenda.erase({p.next_event, w});
    p.next_event = t;
    if (t != kInf) agenda.insert({t, w});
  };
  auto earliest = [&](const Pipe& p) { return p.by_time.empty() ? kInf : std::get<0>(*p.by_time.begin()); };

  for (int32_t i = 0; i < IF; ++i) pipes[0].by_time.insert({0.0, 0, i});
  set_next(0, 0.0);
  int32_t logged = 0;
  while (logged < E) {
    if (agenda.empty()) return -2;
    const int w = agenda.begin()->second;            // lowest time, then lowest pipe index
    Pipe& p = pipes[w];
    // among the events with timestamp <= next_event: best (stage, timestamp, id) by the rule
    auto best = p.by_time.end();
    for (auto it = p.by_time.begin(); it != p.by_time.end() && std::get<0>(*it) <= p.next_event; ++it) {
      if (best == p.by_time.end()) {
        best = it;
        continue;
      }
      const int32_t sa = std::get<1>(*it), sb = std::get<1>(*best);
      const bool better_stage = later_first ? sa > sb : sa < sb;
      // within one stage the set's order (timestamp, then id) already put the right one first
      if (better_stage) best = it;
    }
    if (best == p.by_time.end()) return -2;
    Event ev{std::get<1>(*best), std::get<0>(*best), std::get<2>(*best)};
    p.by_time.erase(best);
    {
      const double e = earliest(p);
      set_next(w, e == kInf ? kInf : std::fmax(p.busy_till, e));
    }
    const double delay = larr[ev.stage % S];
    double finish;
    if (ev.stage % 3 != 2) {
      finish = std::fmax(p.busy_till, ev.ts) + delay;
      p.busy_till = finish;
    } else {
      finish = ev.ts + delay;
    }
    const int32_t stage = (ev.stage + 1) % (S * N);
    const int nw = stage_to_pipe(stage);
    pipes[nw].by_time.insert({finish, stage, ev.id});
    set_next(nw, std::fmax(pipes[nw].busy_till, earliest(pipes[nw])));
    if (stage == 0 && ev.id == 0) gen_ts[logged++] = ev.ts;
  }
  return 0;
}

}  // namespace

extern "C" {

int32_t gh_sim_two_tier(int32_t N, int32_t K, int32_t IF, int32_t E, double t_net_12,
                        double t_net_21, double t_net_rtt, double t_c_att, double t_c_nonatt,
                        int32_t later_first, double* gen_ts) {
  const double larr[6] = {t_c_nonatt, t_net_12, t_net_rtt / 2, t_c_att, t_net_21, t_net_rtt / 2};
  return simulate(larr, 6, N, K, IF, E, later_first != 0, gen_ts);
}

int32_t gh_sim_single_tier(int32_t N, int32_t K, int32_t IF, int32_t E, double t_net_link,
                           double t_net_rtt, double t_c, int32_t later_first, double* gen_ts) {
  const double larr[3] = {t_c, t_net_link, t_net_rtt / 2};
  return simulate(larr, 3, N, K, IF, E, later_first != 0, gen_ts);
}

double gh_sim_tbt(const double* gen_ts, int32_t E, int32_t warmup) {
  if (!gen_ts || warmup < 0 || E < warmup + 2) return -1.0;
  return (gen_ts[E - 1] - gen_ts[warmup]) / (double)(E - 1 - warmup);
}

int32_t gh_sim_if_pp(int32_t K, int32_t N, double t_n, double t_c) {
  return (int32_t)std::ceil(1.0 + (double)K * t_n / ((double)N * t_c)) * K;
}

int32_t gh_sim_if_gh(double t_c2_att, double t_n, double t_c1_noatt) {
  return (int32_t)std::ceil(1.0 + (t_c2_att + t_n) / t_c1_noatt);
}

int32_t gh_sim_if_tp(int32_t K, double t_n, double t_c_min) {
  return (int32_t)std::ceil(1.0 + t_n / (t_c_min / (double)K));
}

int64_t gh_sim_max_batch(double C_max, double M, int32_t n_in_flight) {
  if (M <= 0 || n_in_flight <= 0) return 0;
  return (int64_t)std::floor(C_max / (M * (double)n_in_flight));
}

}  // extern "C"

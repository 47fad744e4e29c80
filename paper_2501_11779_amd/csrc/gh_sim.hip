// Discrete-event simulation of the single-tier and two-tier pipelines (host code only).
// Contract and the passages followed: include/gh_sim.h.
//
// The model: every Tier-1 node owns one station per stage kind of a layer.  A station is either a
// server (a compute node or a link: one batch at a time, the others wait) or a delay (half a round
// trip: any number of batches at once).  A batch is a job that hops from station to station; the
// station whose decision is due first chooses among the jobs that have reached it.  Waiting jobs
// are kept ordered by arrival time, so a decision looks only at the jobs that have arrived, and
// the stations' decision times sit in one ordered agenda instead of being scanned.
#include "gh_sim.h"

#include <cmath>
#include <limits>
#include <set>
#include <tuple>
#include <vector>

namespace {

constexpr double kNever = std::numeric_limits<double>::infinity();

struct StageKind {
  double latency;
  bool server;        // false: a pure delay
};

struct Job {
  double arrival;
  int32_t hop;        // stages gone through since the first layer of the pass
  int32_t batch;
  bool operator<(const Job& o) const {
    return std::tie(arrival, hop, batch) < std::tie(o.arrival, o.hop, o.batch);
  }
};

class Station {
 public:
  StageKind kind{0.0, true};
  double decide_at = kNever;          // when the next job is chosen; kNever: nothing waits

  double first_arrival() const { return waiting_.empty() ? kNever : waiting_.begin()->arrival; }

  // A job arrives: the decision is due once the station is free and something has arrived.
  void accept(const Job& j) {
    waiting_.insert(j);
    decide_at = std::fmax(free_at_, first_arrival());
  }

  // Among the jobs that have arrived by the decision time: the one furthest along (or least far),
  // then the earliest arrival, then the lowest batch.  The next decision is scheduled from the
  // state before the chosen job occupies the station (see gh_sim.h), i.e. before serve().
  bool choose(bool further_along_first, Job* out) {
    auto best = waiting_.end();
    for (auto it = waiting_.begin(); it != waiting_.end() && it->arrival <= decide_at; ++it) {
      // within one hop count the set's order (arrival, then batch) already put the right one first
      if (best == waiting_.end() || (further_along_first ? it->hop > best->hop : it->hop < best->hop))
        best = it;
    }
    if (best == waiting_.end()) return false;
    *out = *best;
    waiting_.erase(best);
    const double next = first_arrival();
    decide_at = next == kNever ? kNever : std::fmax(free_at_, next);
    return true;
  }

  // Departure time of a job that arrived at `arrival`.
  double serve(double arrival) {
    if (!kind.server) return arrival + kind.latency;
    free_at_ = std::fmax(free_at_, arrival) + kind.latency;
    return free_at_;
  }

 private:
  std::set<Job> waiting_;
  double free_at_ = 0.0;
};

// kinds: the stages of one layer in order.  passes: E times at which batch 0 entered the last
// stage of a pass over all N layers.
int32_t simulate(const std::vector<StageKind>& kinds, int32_t N, int32_t K, int32_t IF, int32_t E,
                 bool further_along_first, double* passes) {
  if (!passes) return -1;
  if (N <= 0 || K <= 0 || IF <= 0 || E <= 0 || N % K != 0) return -2;
  const int per_layer = (int)kinds.size();
  const int layers_per_node = N / K;
  const int32_t hops_per_pass = per_layer * N;
  std::vector<Station> stations((size_t)per_layer * K);
  for (size_t i = 0; i < stations.size(); ++i) stations[i].kind = kinds[i % per_layer];
  std::set<std::pair<double, int>> agenda;            // (decision time, station), finite times only
  auto station_of = [&](int32_t hop) { return (hop / per_layer) / layers_per_node * per_layer + hop % per_layer; };
  // runs `change` on station i and keeps the agenda in step with its decision time
  auto update = [&](int i, auto&& change) {
    Station& st = stations[i];
    if (st.decide_at != kNever) agenda.erase({st.decide_at, i});
    change(st);
    if (st.decide_at != kNever) agenda.insert({st.decide_at, i});
  };

  for (int32_t b = 0; b < IF; ++b) update(0, [&](Station& st) { st.accept(Job{0.0, 0, b}); });
  int32_t done = 0;
  while (done < E) {
    if (agenda.empty()) return -2;
    const int i = agenda.begin()->second;               // earliest decision, first station on ties
    Job job{};
    bool chosen = false;
    update(i, [&](Station& st) { chosen = st.choose(further_along_first, &job); });
    if (!chosen) return -2;
    const double leaves = stations[i].serve(job.arrival);
    const int32_t hop = (job.hop + 1) % hops_per_pass;
    update(station_of(hop), [&](Station& st) { st.accept(Job{leaves, hop, job.batch}); });
    if (hop == 0 && job.batch == 0) passes[done++] = job.arrival;
  }
  return 0;
}

}  // namespace

extern "C" {

int32_t gh_sim_two_tier(int32_t N, int32_t K, int32_t IF, int32_t E, double t_net_12,
                        double t_net_21, double t_net_rtt, double t_c_att, double t_c_nonatt,
                        int32_t later_first, double* gen_ts) {
  return simulate({{t_c_nonatt, true}, {t_net_12, true}, {t_net_rtt / 2, false},
                   {t_c_att, true}, {t_net_21, true}, {t_net_rtt / 2, false}},
                  N, K, IF, E, later_first != 0, gen_ts);
}

int32_t gh_sim_single_tier(int32_t N, int32_t K, int32_t IF, int32_t E, double t_net_link,
                           double t_net_rtt, double t_c, int32_t later_first, double* gen_ts) {
  return simulate({{t_c, true}, {t_net_link, true}, {t_net_rtt / 2, false}}, N, K, IF, E,
                  later_first != 0, gen_ts);
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

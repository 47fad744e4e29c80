// Runs the pipeline simulators of csrc/gh_sim.hip (host code only) on configurations read from
// standard input, one per line, and prints the token times as hexadecimal floats, so that a build
// under AddressSanitizer / UndefinedBehaviorSanitizer can be compared with the Python oracle
// (tests/test_sanitized_host_code.py).
//   two    N K IF E t_net_12 t_net_21 t_net_rtt t_c_att t_c_nonatt later_first
//   single N K IF E t_net_link t_net_rtt t_c later_first
#include <cstdio>
#include <cstring>
#include <vector>

#include "../../paper_2501_11779_amd/csrc/gh_sim.hip"

int main() {
  char kind[16];
  while (std::scanf("%15s", kind) == 1) {
    int N, K, IF, E, later;
    double t[5];
    int status;
    std::vector<double> out;
    if (!std::strcmp(kind, "two")) {
      if (std::scanf("%d %d %d %d %lf %lf %lf %lf %lf %d", &N, &K, &IF, &E, &t[0], &t[1], &t[2], &t[3],
                     &t[4], &later) != 10) return 2;
      out.assign(E > 0 ? E : 1, -1.0);
      status = gh_sim_two_tier(N, K, IF, E, t[0], t[1], t[2], t[3], t[4], later, out.data());
    } else {
      if (std::scanf("%d %d %d %d %lf %lf %lf %d", &N, &K, &IF, &E, &t[0], &t[1], &t[2], &later) != 8)
        return 2;
      out.assign(E > 0 ? E : 1, -1.0);
      status = gh_sim_single_tier(N, K, IF, E, t[0], t[1], t[2], later, out.data());
    }
    std::printf("%d", status);
    if (status == 0)
      for (int e = 0; e < E; ++e) std::printf(" %a", out[e]);
    std::printf("\n");
  }
  return 0;
}

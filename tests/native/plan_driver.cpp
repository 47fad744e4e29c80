// Replays the balanced split in host C++ from the library's own planning code (csrc/gh_plan.hpp):
// for every worker the tiles it takes, the strips they fall in and the record index it would
// write, with the arithmetic of the attention kernel (share, first worker of a strip, record =
// worker - first).  Reads problems from standard input and prints, per problem, the plan and the
// number of records of every strip -- or "BAD ..." when an index leaves [0, n_chunks), when a
// strip's records are not numbered 0, 1, 2, ... or when its pieces do not tile it.
//   B H H_kv max_ctx T n_groups rows[0] ... rows[n_groups-1]      (rows: rows streamed per group)
// Compared with the Python emulation of the same split in tests/test_sanitized_host_code.py, and
// built with the sanitizers there.
#include <cstdio>
#include <vector>

#include "../../paper_2501_11779_amd/csrc/gh_plan.hpp"

int main() {
  int B, H, Hkv, max_ctx, T, n_groups;
  while (std::scanf("%d %d %d %d %d %d", &B, &H, &Hkv, &max_ctx, &T, &n_groups) == 6) {
    std::vector<long long> rows(n_groups);
    for (auto& r : rows)
      if (std::scanf("%lld", &r) != 1) return 2;
    gh_problem p{};
    p.batch = B;
    p.n_q_heads = H;
    p.n_kv_heads = Hkv;
    p.head_dim = 128;
    p.dtype = GH_BF16;
    p.n_slots = n_groups > 0 ? n_groups : 1;
    p.slot_capacity = max_ctx;
    p.max_ctx_len = max_ctx;
    p.slot_stride = (int64_t)Hkv * max_ctx * 128;
    p.head_stride = (int64_t)max_ctx * 128;
    p.row_stride = 128;
    p.scale = 0.088f;
    p.tokens_per_group = T;
    const int32_t st = gh_plan::check_problem(&p);
    if (st != GH_OK) {
      std::printf("STATUS %d\n", st);
      continue;
    }
    const gh_plan::Plan pl = gh_plan::make_plan(&p);
    if (!pl.balanced) {
      std::printf("FIXED %d %d\n", pl.chunk_rows, pl.n_chunks);
      continue;
    }
    // strips laid end to end: group, kv head, pass set; every strip of a group has the same tiles
    const long long spb = (long long)Hkv * pl.n_pass;
    std::vector<long long> cum(n_groups + 1, 0);
    for (int g = 0; g < n_groups; ++g) {
      const long long tiles = rows[g] > 0 ? (rows[g] + 31) / 32 : 1;
      cum[g + 1] = cum[g] + tiles * spb;
    }
    const long long total = cum[n_groups];
    long long share = (total + pl.n_workers - 1) / pl.n_workers;
    if (share < pl.min_share) share = pl.min_share;
    std::vector<int> records((size_t)n_groups * spb, 0);
    std::vector<long long> covered((size_t)n_groups * spb, 0);
    bool bad = false;
    int g = 0;
    for (long long w = 0; w < pl.n_workers && !bad; ++w) {
      const long long t0 = w * share, t_end = t0 + share < total ? t0 + share : total;
      if (t0 >= total) break;
      while (cum[g + 1] <= t0) ++g;                               // group of the worker's first tile
      int gg = g;
      long long t = t0;
      while (t < t_end) {
        while (cum[gg + 1] <= t) ++gg;
        const long long tiles = (cum[gg + 1] - cum[gg]) / spb;
        const long long sib = (t - cum[gg]) / tiles;              // strip within the group
        const long long strip_t0 = cum[gg] + sib * tiles;
        const long long piece_end = strip_t0 + tiles < t_end ? strip_t0 + tiles : t_end;
        const long long rec = w - strip_t0 / share;               // the kernel's record index
        const size_t id = (size_t)gg * spb + sib;
        if (rec < 0 || rec >= pl.n_chunks || rec != records[id] || t - strip_t0 != covered[id]) {
          std::printf("BAD worker %lld strip %zu rec %lld records %d n_chunks %d\n", w, id, rec,
                      records[id], pl.n_chunks);
          bad = true;
          break;
        }
        ++records[id];
        covered[id] += piece_end - t;
        t = piece_end;
      }
    }
    if (bad) continue;
    std::printf("PLAN %d %d %d %d %d %d %lld", pl.n_workers, pl.min_share, pl.passes_per_strip,
                pl.share, pl.n_pass, pl.n_chunks, share);
    for (size_t i = 0; i < records.size(); ++i) {
      const long long tiles = (cum[i / spb + 1] - cum[i / spb]) / spb;
      if (covered[i] != tiles) {
        std::printf(" UNCOVERED %zu", i);
        break;
      }
      std::printf(" %d", records[i]);
    }
    std::printf("\n");
  }
  return 0;
}

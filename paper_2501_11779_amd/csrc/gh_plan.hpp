// Host-side judgement of a gh_problem and the launch plan derived from it: plain C++ with no HIP
// in it, so that it also compiles (and runs under the sanitizers) on a machine without a GPU.
// Included by gh_tier2.hip; the contract of every number here is in include/gh_tier2.h.
#pragma once
#include <stddef.h>
#include <stdint.h>

#include "gh_tier2.h"

namespace gh_plan {

constexpr int kHeadDim = 128;

constexpr int kComputeUnits = 256;          // MI355X
constexpr int kChunkQuantum = 64;           // chunk_rows granularity
constexpr int kMinAutoChunk = 256;

inline int round_up(int x, int q) { return (x + q - 1) / q * q; }

// Blocked-layout parameters for the kernels; a plain layout is one block holding every row.
inline void block_params(const gh_problem* p, int64_t* stride, int32_t* shift, int32_t* mask) {
  if (p->block_rows > 0) {
    int s = 0;
    while ((1 << s) < p->block_rows) ++s;
    *shift = s;
    *mask = p->block_rows - 1;
    *stride = p->block_stride;
  } else {
    *shift = 31;
    *mask = 0x7fffffff;
    *stride = 0;
  }
}

inline bool aligned16(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

constexpr int kBalancedMaxBatch = 4096;     // groups per launch of the balanced split: three
                                            // per-group arrays live in LDS (48 KB); a larger batch
                                            // is launched in slices
constexpr int kMaxTokensPerGroup = 64;

inline int tokens_per_group(const gh_problem* p) { return p->tokens_per_group > 1 ? p->tokens_per_group : 1; }

// Everything about gh_problem that can be judged on the host.
inline int32_t check_problem(const gh_problem* p) {
  if (!p) return GH_ERR_NULL;
  if (p->batch < 0 || p->n_q_heads <= 0 || p->n_kv_heads <= 0 || p->n_slots <= 0 ||
      p->slot_capacity <= 0 || p->max_ctx_len < 0)
    return GH_ERR_SHAPE;
  if (p->n_q_heads % p->n_kv_heads != 0) return GH_ERR_SHAPE;
  if (p->head_dim != kHeadDim) return GH_ERR_UNSUPPORTED;
  if (p->dtype != GH_F16 && p->dtype != GH_BF16) return GH_ERR_UNSUPPORTED;
  if (p->kernel != GH_KERNEL_AUTO && p->kernel != GH_KERNEL_VALU && p->kernel != GH_KERNEL_MFMA &&
      p->kernel != GH_KERNEL_STRIPS)
    return GH_ERR_UNSUPPORTED;
  if (p->row_stride < p->head_dim || p->head_stride <= 0 || p->slot_stride <= 0) return GH_ERR_SHAPE;
  if (p->row_stride % 8 || p->head_stride % 8 || p->slot_stride % 8) return GH_ERR_UNSUPPORTED;
  // the kernels form a row's byte offset inside a 32-row tile with 24-bit multiplies
  if (p->row_stride >= (1 << 22)) return GH_ERR_UNSUPPORTED;
  if (p->max_ctx_len > p->slot_capacity) return GH_ERR_CAPACITY;
  if (p->chunk_rows < 0 || p->chunk_rows % kChunkQuantum != 0) return GH_ERR_SHAPE;
  if (p->block_rows < 0 || (p->block_rows > 0 && p->block_stride <= 0)) return GH_ERR_SHAPE;
  if (p->block_rows > 0 && (p->block_rows < 32 || (p->block_rows & (p->block_rows - 1)) != 0))
    return GH_ERR_UNSUPPORTED;
  if (p->block_rows > 0 && p->block_stride % 8) return GH_ERR_UNSUPPORTED;
  if (p->tokens_per_group < 0) return GH_ERR_SHAPE;
  if (p->tokens_per_group > 1) {
    // groups run on the matrix-core kernel with the library's split only
    if (p->batch % p->tokens_per_group != 0) return GH_ERR_SHAPE;
    if (p->tokens_per_group > kMaxTokensPerGroup || p->kernel == GH_KERNEL_VALU ||
        p->chunk_rows != 0)
      return GH_ERR_UNSUPPORTED;
  }
  if (p->q_batch_stride < 0 || p->new_batch_stride < 0) return GH_ERR_SHAPE;
  if (p->q_batch_stride % 8 || p->new_batch_stride % 8) return GH_ERR_UNSUPPORTED;
  if (p->q_batch_stride != 0 && p->q_batch_stride < (int64_t)p->n_q_heads * p->head_dim)
    return GH_ERR_SHAPE;
  if (p->new_batch_stride != 0 && p->new_batch_stride < (int64_t)p->n_kv_heads * p->head_dim)
    return GH_ERR_SHAPE;
  return GH_OK;
}

inline int resolve_kernel(const gh_problem* p) {
  // Measured on MI355X: the matrix-core kernel is faster for every head-group size, plain
  // multi-head attention included (81% against 68% of peak HBM bandwidth at group size 1).
  // (GH_KERNEL_STRIPS only changes gh_decode_step; everywhere else it is the matrix-core kernel)
  return p->kernel == GH_KERNEL_VALU ? GH_KERNEL_VALU : GH_KERNEL_MFMA;
}

// Heads of one kv head handled by a single work item, and how many such passes.
inline void head_passes(const gh_problem* p, int kernel, int* per_pass, int* n_pass) {
  // head columns of one (group, kv head): the G heads of each of the group's token rows
  const int group = p->n_q_heads / p->n_kv_heads * tokens_per_group(p);
  int hp;
  if (kernel == GH_KERNEL_MFMA) {
    hp = 16;
  } else {
    hp = group > 4 ? 8 : group > 2 ? 4 : group;    // 1, 2, 4 or 8
  }
  *per_pass = hp;
  *n_pass = (group + hp - 1) / hp;
}

// Rows per chunk: the largest multiple of the quantum that still gives the
// chip a few work items per wave slot, but not below kMinAutoChunk rows.
inline int auto_chunk_rows(const gh_problem* p) {
  const int whole = round_up(p->max_ctx_len > 0 ? p->max_ctx_len : 1, kChunkQuantum);
  int per_pass, n_pass;
  head_passes(p, resolve_kernel(p), &per_pass, &n_pass);
  const int64_t strips = (int64_t)(p->batch > 0 ? p->batch : 1) * p->n_kv_heads * n_pass;
  const int64_t want_items = (int64_t)kComputeUnits * 32;
  int64_t chunks = (want_items + strips - 1) / strips;       // chunks per strip wanted
  if (chunks < 1) chunks = 1;
  int rows = round_up((int)((whole + chunks - 1) / chunks), kChunkQuantum);
  if (rows < kMinAutoChunk) rows = kMinAutoChunk;
  if (rows > whole) rows = whole;
  return rows;
}

struct Plan {
  int kernel, chunk_rows, n_chunks, per_pass, n_pass;
  bool balanced;            // equal shares of 32-row tiles per wave instead of fixed chunks
  int n_workers, min_share; // balanced split only
  int passes_per_strip;     // balanced split: passes a wave carries through a strip at once;
                            // n_pass then counts strips per (group, kv head)
  int share;                // balanced split: waves per worker (1, or 4: a whole workgroup); the
                            // waves of a worker walk the same tiles, each with its own
                            // passes_per_strip passes
  int launch_groups;        // balanced split: groups per launch (the batch goes in slices of
                            // this many groups, each split on its own)
};

constexpr int kBalancedWavesPerCU = 4;      // waves of the balanced kernel per compute unit: one per
                                            // SIMD (measured against two: 0.2-2% faster on the large
                                            // workloads, 6-13% on batches of 16 to 64 sequences)
constexpr int kBalancedMaxRecords = 64;     // partial records per (sequence, head)

inline Plan make_plan(const gh_problem* p) {
  Plan pl;
  pl.kernel = resolve_kernel(p);
  head_passes(p, pl.kernel, &pl.per_pass, &pl.n_pass);
  pl.balanced = false;
  pl.n_workers = pl.min_share = 0;
  pl.passes_per_strip = 1;
  pl.share = 1;
  pl.launch_groups = 0;
  const int all_groups = p->batch / tokens_per_group(p);
  const int groups = all_groups < kBalancedMaxBatch ? all_groups : kBalancedMaxBatch;   // of one launch
  // Head columns per kv head (a head group, or a token group's heads) in passes of 16:
  //   up to 16: a wave carries one pass;
  //   up to 32: a wave carries two passes through one stream of tiles, at one wave per SIMD (the
  //             second pass's operands and accumulators take the other wave's registers);
  //   more:     the four waves of a workgroup form one worker that streams the tiles once -- each
  //             wave fetches a quarter, they put the tile together in LDS and read their operands
  //             from there -- with one pass per wave (up to 64 columns) or two (up to 128 columns
  //             per strip), two workgroups per compute unit.  K/V rows are read from memory once
  //             per 128 head columns.
  const int pps = pl.n_pass == 2 || pl.n_pass > 4 ? 2 : 1;
  const int share = pl.n_pass > 2 ? 4 : 1;
  const int sets = (pl.n_pass + pps - 1) / pps;
  const int n_strip = (sets + share - 1) / share;
  const int64_t strips = (int64_t)(groups > 0 ? groups : 1) * p->n_kv_heads * n_strip;
  // (+ 1: the one-launch step walks the appended row as a tile of its own behind the cached rows)
  const int64_t max_tiles = (p->max_ctx_len > 0 ? (p->max_ctx_len + 31) / 32 : 1) + 1;
  if (pl.kernel == GH_KERNEL_MFMA && p->chunk_rows == 0 && strips * max_tiles < 0x7fffffff) {
    // Records per head: enough for the longest strip when strips are up to four times the
    // average length; beyond that the share per wave grows instead (min_share).
    pl.balanced = true;
    pl.passes_per_strip = pps;
    pl.n_pass = n_strip;
    pl.share = share;
    pl.launch_groups = groups > 0 ? groups : 1;
    // workers: a wave each, one per SIMD; or a workgroup each, two per compute unit
    pl.n_workers = share == 4 ? kComputeUnits * 2 : kComputeUnits * kBalancedWavesPerCU;
    int64_t c = (4 * (int64_t)pl.n_workers + strips - 1) / strips + 1;
    if (c < 2) c = 2;
    if (c > kBalancedMaxRecords) c = kBalancedMaxRecords;
    if (c > max_tiles + 1) c = max_tiles + 1;
    pl.n_chunks = (int)c;
    pl.min_share = (int)((max_tiles + pl.n_chunks - 2) / (pl.n_chunks - 1));
    pl.chunk_rows = 0;
    return pl;
  }
  pl.chunk_rows = p->chunk_rows > 0 ? p->chunk_rows : auto_chunk_rows(p);
  pl.n_chunks = p->max_ctx_len > 0 ? (p->max_ctx_len + pl.chunk_rows - 1) / pl.chunk_rows : 1;
  return pl;
}

// o, m, l of every record, the record counts, and the arrival counters of the one-launch step
// (one per strip; there are never more strips than heads)
inline size_t workspace_floats(const gh_problem* p, const Plan& pl) {
  return (size_t)p->batch * p->n_q_heads * ((size_t)pl.n_chunks * (kHeadDim + 2) + 2);
}

}  // namespace gh_plan

// Merge of the per-chunk partial softmax results into the final output.
#pragma once
#include "gh_common.hpp"

namespace gh {

struct ReduceArgs {
  const float* ws_o;   // [B*H, C, 128]
  const float* ws_m;   // [B*H, C]
  const float* ws_l;   // [B*H, C]
  const int32_t* ws_n; // [B*H]  records in use
  float* out;          // [B*H, 128]
  int64_t n_rows;      // B * H
  int32_t n_chunks;
};

// One wave per (sequence, head); a lane owns two adjacent columns.  Chunks are
// visited in index order, so the result does not depend on scheduling.
__global__ __launch_bounds__(256) void decode_reduce_kernel(const ReduceArgs a) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= a.n_rows) return;
  const float* m = a.ws_m + row * a.n_chunks;
  const float* l = a.ws_l + row * a.n_chunks;
  const float* o = a.ws_o + row * a.n_chunks * kHeadDim + 2 * lane;
  int used = a.ws_n[row];
  used = used < 0 ? 0 : used < a.n_chunks ? used : a.n_chunks;
  float M = kNegInf;
  for (int c = 0; c < used; ++c)
    if (l[c] > 0.f) M = fmaxf(M, m[c]);
  float2 acc = make_float2(0.f, 0.f);
  float L = 0.f;
  if (M != kNegInf) {
    for (int c = 0; c < used; ++c) {
      const float lc = l[c];
      if (!(lc > 0.f)) continue;                     // empty chunk: its o is unspecified
      const float w = fast_exp2(m[c] - M);
      const float2 oc = *reinterpret_cast<const float2*>(o + (int64_t)c * kHeadDim);
      acc.x = fmaf(w, oc.x, acc.x);
      acc.y = fmaf(w, oc.y, acc.y);
      L = fmaf(w, lc, L);
    }
    acc.x /= L;
    acc.y /= L;
  }
  *reinterpret_cast<float2*>(a.out + row * kHeadDim + 2 * lane) = acc;
}

}  // namespace gh

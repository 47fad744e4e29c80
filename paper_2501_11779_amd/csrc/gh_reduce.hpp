// Merge of the per-chunk partial softmax results into the final output.
#pragma once
#include "gh_common.hpp"

namespace gh {

struct ReduceArgs {
  const float* ws_o;   // [B*H, C, 128]
  const float* ws_m;   // [B*H, C]
  const float* ws_l;   // [B*H, C]
  const int32_t* ws_n; // [B*H]  records in use
  void* out;           // [B*H, 128] fp32, or the 16-bit model type
  int64_t n_rows;      // B * H
  int32_t n_chunks;
};

__device__ __forceinline__ float wave_max(float x) {
#pragma unroll
  for (int off = 32; off >= 1; off >>= 1) x = fmaxf(x, __shfl_xor(x, off, 64));
  return x;
}

// One wave per (sequence, head); a lane owns two adjacent columns.  Heads with at most two records
// take a short path on prefetched values; otherwise the (m, l) of the records are read 64 at a
// time, one per lane, to find the common maximum and the weights, and the o rows are accumulated in
// record order with independent loads.  Either way the order of the arithmetic is fixed, so the
// result does not depend on scheduling.
// OUT: 0 = fp32, 1 = binary16, 2 = bfloat16 (round to nearest even at the store).
template <int OUT>
__global__ __launch_bounds__(256) void decode_reduce_kernel(const ReduceArgs a) {
  const int lane = threadIdx.x & 63;
  const int64_t row = (int64_t)blockIdx.x * 4 + (threadIdx.x >> 6);
  if (row >= a.n_rows) return;
  const float* m = a.ws_m + row * a.n_chunks;
  const float* l = a.ws_l + row * a.n_chunks;
  const float* o = a.ws_o + row * a.n_chunks * kHeadDim + 2 * lane;

  // A row that the attention kernel has stored already needs nothing: the count says so, and is
  // read first (on batches where most rows are such, fetching records ahead of it was a third of
  // this kernel's time: 16.8 -> 12.1 us on 65 536 rows of which three in four were done).
  int used = a.ws_n[row];
  if (used < 0) return;
  // The first two records are fetched before the count is looked at further: they exist in the
  // layout whatever it says, most heads use one or two, and the headers and the rows then cost one
  // more memory round trip instead of two.  What a record beyond the count holds is never used.
  const bool two = a.n_chunks > 1;
  const float2 o0 = *reinterpret_cast<const float2*>(o);
  const float2 o1 = two ? *reinterpret_cast<const float2*>(o + kHeadDim) : make_float2(0.f, 0.f);
  const float m0 = m[0], l0 = l[0];
  const float m1 = two ? m[1] : kNegInf, l1 = two ? l[1] : 0.f;
  // ... and so are the headers of the first 64 records, one per lane, for heads with more
  const int ch = lane < a.n_chunks ? lane : 0;
  const float mh = m[ch], lh = l[ch];
  used = used < a.n_chunks ? used : a.n_chunks;

  float2 acc = make_float2(0.f, 0.f);
  if (used <= 2) {
    const float la = used > 0 ? l0 : 0.f, lb = used > 1 ? l1 : 0.f;
    const float ma = la > 0.f ? m0 : kNegInf, mb = lb > 0.f ? m1 : kNegInf;
    const float M = fmaxf(ma, mb);
    if (M != kNegInf) {
      const float wa = la > 0.f ? fast_exp2(ma - M) : 0.f;
      const float wb = lb > 0.f ? fast_exp2(mb - M) : 0.f;
      float L = 0.f;
      if (wa > 0.f) {
        acc.x = fmaf(wa, o0.x, acc.x);
        acc.y = fmaf(wa, o0.y, acc.y);
      }
      L += wa * la;
      if (wb > 0.f) {
        acc.x = fmaf(wb, o1.x, acc.x);
        acc.y = fmaf(wb, o1.y, acc.y);
      }
      L += wb * lb;
      acc.x /= L;
      acc.y /= L;
    }
  } else {
    float M = kNegInf;
    for (int c0 = 0; c0 < used; c0 += 64) {
      const int c = c0 + lane;
      const float lc = c >= used ? 0.f : c0 == 0 ? lh : l[c];
      const float mc = c >= used ? kNegInf : c0 == 0 ? mh : m[c];
      M = fmaxf(M, lc > 0.f ? mc : kNegInf);     // a record without rows carries no maximum
    }
    M = wave_max(M);
    float L = 0.f;
    if (M != kNegInf) {
      for (int c0 = 0; c0 < used; c0 += 64) {
        const int c = c0 + lane;
        const float lc = c >= used ? 0.f : c0 == 0 ? lh : l[c];
        const float mc = c >= used ? kNegInf : c0 == 0 ? mh : m[c];
        const float w = lc > 0.f ? fast_exp2(mc - M) : 0.f;   // this lane's record weight
        const float wl = w * lc;
        const int n = used - c0 < 64 ? used - c0 : 64;
        int j = 0;
        for (; j + 4 <= n; j += 4) {                           // four independent row loads
          float2 oc[4];
          float wj[4];
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            wj[u] = __shfl(w, j + u, 64);
            oc[u] = *reinterpret_cast<const float2*>(o + (int64_t)(c0 + j + u) * kHeadDim);
          }
#pragma unroll
          for (int u = 0; u < 4; ++u) {
            if (wj[u] > 0.f) {                                 // an empty record's o is unspecified
              acc.x = fmaf(wj[u], oc[u].x, acc.x);
              acc.y = fmaf(wj[u], oc[u].y, acc.y);
            }
            L += __shfl(wl, j + u, 64);
          }
        }
        for (; j < n; ++j) {
          const float wj = __shfl(w, j, 64);
          const float2 oc = *reinterpret_cast<const float2*>(o + (int64_t)(c0 + j) * kHeadDim);
          if (wj > 0.f) {
            acc.x = fmaf(wj, oc.x, acc.x);
            acc.y = fmaf(wj, oc.y, acc.y);
          }
          L += __shfl(wl, j, 64);
        }
      }
      acc.x /= L;
      acc.y /= L;
    }
  }
  if constexpr (OUT == 0) {
    *reinterpret_cast<float2*>(static_cast<float*>(a.out) + row * kHeadDim + 2 * lane) = acc;
  } else if constexpr (OUT == 1) {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    const h2 v = {(_Float16)acc.x, (_Float16)acc.y};
    reinterpret_cast<h2*>(a.out)[row * (kHeadDim / 2) + lane] = v;
  } else {
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    const b2 v = {(__bf16)acc.x, (__bf16)acc.y};
    reinterpret_cast<b2*>(a.out)[row * (kHeadDim / 2) + lane] = v;
  }
}

}  // namespace gh

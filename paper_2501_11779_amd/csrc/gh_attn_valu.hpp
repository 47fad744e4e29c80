// Split-context decode attention on the fp32 vector ALUs.
//
// One workgroup (4 waves) owns one (sequence, kv head, head pass, chunk).  A
// wave is 4 rows x 16 lanes: each lane reads 16 bytes (8 columns) of a K or V
// row, so one wave-wide load covers 4 consecutive 256-byte rows = 1 KiB of
// contiguous memory.  The 16 lane-rows of the workgroup walk the chunk with a
// stride of 16 rows, UNROLL rows deep, each keeping its own running
// (max, sum, o[8 columns]) per query head; K and V rows are read once and
// used for all GT heads of the pass.  At the end the 16 running states are
// merged (shuffles inside a wave, LDS across waves) into one partial record.
#pragma once
#include "gh_common.hpp"

namespace gh {

template <int GT, bool BF16>
__global__ __launch_bounds__(256) void attn_valu_kernel(const AttnArgs a) {
  constexpr int UNROLL = 4;
  __shared__ float lds_o[4][GT][kHeadDim];
  __shared__ float lds_m[4][GT];
  __shared__ float lds_l[4][GT];

  const Item it = decode_item(a, blockIdx.x);
  const int tid = threadIdx.x;
  if (it.chunk == 0 && tid < it.nh)          // every record of a head is written in this split
    a.ws_n[(int64_t)it.b * a.n_q_heads + it.h0 + tid] = a.n_chunks;
  if (it.r1 <= it.r0) {                      // empty chunk: flag it and leave
    if (tid < it.nh) {
      const int64_t pi = partial_index(a, it, it.h0 + tid);
      a.ws_m[pi] = kNegInf;
      a.ws_l[pi] = 0.f;
    }
    return;
  }
  const int lane = tid & 63, wave = tid >> 6;
  const int j = lane & 15;                   // 16-byte column chunk: columns 8j .. 8j+7
  const int rg = wave * 4 + (lane >> 4);     // row group 0..15

  // q of the pass, pre-multiplied by scale*log2(e); absent heads are zero.
  float qf[GT][8];
#pragma unroll
  for (int i = 0; i < GT; ++i) {
    if (i < it.nh) {
      const uint4 w = *reinterpret_cast<const uint4*>(
          a.q + (int64_t)it.b * a.q_batch_stride + (it.h0 + i) * kHeadDim + 8 * j);
      unpack8<BF16>(w, qf[i]);
#pragma unroll
      for (int e = 0; e < 8; ++e) qf[i][e] *= a.scale_log2e;
    } else {
#pragma unroll
      for (int e = 0; e < 8; ++e) qf[i][e] = 0.f;
    }
  }

  float m[GT], l[GT], o[GT][8];
#pragma unroll
  for (int i = 0; i < GT; ++i) {
    m[i] = kNegInf;
    l[i] = 0.f;
#pragma unroll
    for (int e = 0; e < 8; ++e) o[i][e] = 0.f;
  }

  const uint16_t* kbase = a.k_cache + it.strip + 8 * j;
  const uint16_t* vbase = a.v_cache + it.strip + 8 * j;
  const int last = it.r1 - 1;

  // The first row of every trip is inside the chunk, so each trip sees a finite score.
  for (int r = it.r0 + rg; r < it.r1; r += 16 * UNROLL) {
    uint4 kw[UNROLL], vw[UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      const int row = r + 16 * u;
      const int64_t off = row_offset(row < last ? row : last, a.row_stride, a.block_stride,
                                     a.block_shift, a.block_mask);
      kw[u] = __builtin_bit_cast(uint4, stream_load(kbase + off));
      vw[u] = __builtin_bit_cast(uint4, stream_load(vbase + off));
    }
    float s[GT][UNROLL];
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      float kf[8];
      unpack8<BF16>(kw[u], kf);
      const bool live = r + 16 * u < it.r1;
#pragma unroll
      for (int i = 0; i < GT; ++i) {
        float acc = qf[i][0] * kf[0];
#pragma unroll
        for (int e = 1; e < 8; ++e) acc = fmaf(qf[i][e], kf[e], acc);
        acc = row16_sum(acc);
        s[i][u] = live ? acc : kNegInf;
      }
    }
    float alpha[GT];
#pragma unroll
    for (int i = 0; i < GT; ++i) {
      float mx = s[i][0];
#pragma unroll
      for (int u = 1; u < UNROLL; ++u) mx = fmaxf(mx, s[i][u]);
      const float mn = fmaxf(m[i], mx);
      alpha[i] = fast_exp2(m[i] - mn);
      m[i] = mn;
      float sum = 0.f;
#pragma unroll
      for (int u = 0; u < UNROLL; ++u) {
        s[i][u] = fast_exp2(s[i][u] - mn);
        sum += s[i][u];
      }
      l[i] = fmaf(l[i], alpha[i], sum);
#pragma unroll
      for (int e = 0; e < 8; ++e) o[i][e] *= alpha[i];
    }
#pragma unroll
    for (int u = 0; u < UNROLL; ++u) {
      float vf[8];
      unpack8<BF16>(vw[u], vf);
#pragma unroll
      for (int i = 0; i < GT; ++i)
#pragma unroll
        for (int e = 0; e < 8; ++e) o[i][e] = fmaf(s[i][u], vf[e], o[i][e]);
    }
  }

  // Merge the four lane-rows of the wave.
#pragma unroll
  for (int i = 0; i < GT; ++i) {
    float M = fmaxf(m[i], xor16(m[i]));
    M = fmaxf(M, xor32(M));
    const float w = m[i] == kNegInf ? 0.f : fast_exp2(m[i] - M);
    float ll = l[i] * w;
    ll += xor16(ll);
    ll += xor32(ll);
    l[i] = ll;
    m[i] = M;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float x = o[i][e] * w;
      x += xor16(x);
      x += xor32(x);
      o[i][e] = x;
    }
  }
  if (lane < 16) {
#pragma unroll
    for (int i = 0; i < GT; ++i) {
#pragma unroll
      for (int e = 0; e < 8; ++e) lds_o[wave][i][8 * j + e] = o[i][e];
      if (j == 0) {
        lds_m[wave][i] = m[i];
        lds_l[wave][i] = l[i];
      }
    }
  }
  __syncthreads();

  // Merge the four waves and write the partial record: thread -> (head, column).
  for (int idx = tid; idx < GT * kHeadDim; idx += 256) {
    const int i = idx / kHeadDim, col = idx % kHeadDim;
    if (i >= it.nh) continue;
    float M = kNegInf;
#pragma unroll
    for (int w = 0; w < 4; ++w) M = fmaxf(M, lds_m[w][i]);
    float acc = 0.f, L = 0.f;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const float mw = lds_m[w][i];
      const float f = mw == kNegInf ? 0.f : fast_exp2(mw - M);
      acc = fmaf(f, lds_o[w][i][col], acc);
      L = fmaf(f, lds_l[w][i], L);
    }
    const int64_t pi = partial_index(a, it, it.h0 + i);
    a.ws_o[pi * kHeadDim + col] = acc;
    if (col == 0) {
      a.ws_m[pi] = M;
      a.ws_l[pi] = L;
    }
  }
}

}  // namespace gh

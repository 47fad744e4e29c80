// Append of the step's new key/value rows into the context slots: a bit copy.
#pragma once
#include "gh_common.hpp"

namespace gh {

struct AppendArgs {
  uint16_t* k_cache;
  uint16_t* v_cache;
  const uint16_t* k_new;     // [B, H_kv, 128]
  const uint16_t* v_new;
  const int32_t* slot_id;    // [B]
  const int32_t* pos;        // [B]
  int32_t* dev_status;       // nullable
  int64_t slot_stride, head_stride, row_stride;
  int64_t new_batch_stride;  // elements between sequences in k_new / v_new
  int64_t block_stride;      // blocked layout, see row_offset()
  int32_t block_shift, block_mask;
  int32_t batch, n_kv_heads, n_slots, capacity;
};

// One thread moves 16 bytes: 16 threads per row, K rows then V rows of a (sequence, kv head).
__global__ __launch_bounds__(256) void kv_append_kernel(const AppendArgs a) {
  const int64_t t = (int64_t)blockIdx.x * 256 + threadIdx.x;
  const int j = (int)(t & 15);
  const int which = (int)((t >> 4) & 1);
  const int64_t pair = t >> 5;                       // b * H_kv + g
  if (pair >= (int64_t)a.batch * a.n_kv_heads) return;
  const int b = (int)(pair / a.n_kv_heads), g = (int)(pair % a.n_kv_heads);
  const int slot = a.slot_id[b], p = a.pos[b];
  const bool bad_slot = slot < 0 || slot >= a.n_slots;
  const bool bad_pos = p < 0 || p >= a.capacity;
  if (bad_slot || bad_pos) {
    if (a.dev_status && g == 0 && j == 0 && which == 0)
      atomicOr(a.dev_status, (bad_slot ? 1 : 0) | (bad_pos ? 2 : 0));
    return;
  }
  const int64_t dst = (int64_t)slot * a.slot_stride + (int64_t)g * a.head_stride +
                      row_offset(p, a.row_stride, a.block_stride, a.block_shift, a.block_mask) + 8 * j;
  const int64_t src = (int64_t)b * a.new_batch_stride + g * kHeadDim + 8 * j;
  const uint16_t* from = which ? a.v_new : a.k_new;
  uint16_t* to = which ? a.v_cache : a.k_cache;
  *reinterpret_cast<uint4*>(to + dst) = *reinterpret_cast<const uint4*>(from + src);
}

}  // namespace gh

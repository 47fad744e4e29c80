// Shared device-side definitions of the Tier-2 attention kernels (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gh {

constexpr int kHeadDim = 128;        // columns per K/V row
constexpr int kRowBytes = 256;       // head_dim * 2 bytes
constexpr float kNegInf = -__builtin_huge_valf();

// Arguments of both attention kernels (passed by value).
struct AttnArgs {
  const uint16_t* q;        // [B, H, 128]
  const uint16_t* k_cache;
  const uint16_t* v_cache;
  const int32_t* slot_id;   // [B]
  const int32_t* ctx_len;   // [B]
  float* ws_o;              // [B, H, C, 128]
  float* ws_m;              // [B, H, C]
  float* ws_l;              // [B, H, C]
  int32_t* ws_n;            // [B, H]  records in use per head
  int64_t slot_stride, head_stride, row_stride;   // elements
  int64_t q_batch_stride;                         // elements between sequences in q
  int64_t block_stride;                           // blocked layout, see row_offset()
  int32_t block_shift, block_mask;                // log2(block_rows), block_rows - 1
  int32_t n_q_heads, n_kv_heads;                  // H, H_kv
  int32_t tokens, real_group;                     // T token rows per group, G = H / H_kv
  int32_t group;                                  // head columns per (group, kv head): T * G
  int32_t n_slots, row_limit;                     // row_limit = min(capacity, max_ctx_len)
  int32_t chunk_rows, n_chunks;
  int32_t heads_per_pass, n_pass;                 // head sub-groups of one kv head
  int32_t n_items;                                // B * H_kv * n_pass * n_chunks (fixed split)
  int32_t batch;
  int32_t n_workers, min_share;                   // balanced split: workers, least tiles per worker
  int32_t share;                                  // balanced split: waves per worker (1, or 4: a workgroup)
  float scale_log2e;                              // scale * log2(e)
  void* out;                                      // final results of heads one wave covers alone
  int32_t out_kind;                               // 0 none, 1 fp32, 2 binary16, 3 bfloat16
  // The whole step in one launch (gh_decode_step): ctx_len[] then holds the positions of the new
  // rows (rows attended = position + 1, ctx_bias = 1), the new rows are taken from k_new / v_new
  // and written into the caches by the wave that reaches them, and the wave that delivers the
  // last record of a strip merges the strip's records (arrival counters, zero between launches).
  int32_t ctx_bias;                               // 0, or 1 when ctx_len[] holds positions
  const uint16_t* k_new;                          // [B, H_kv, 128]
  const uint16_t* v_new;
  int64_t new_batch_stride;                       // elements between sequences in k_new / v_new
  int32_t* arrive;                                // [B * H_kv * n_pass]
  int32_t* dev_status;                            // nullable
};

// Clears n 32-bit words (a kernel, not a memset: it can be captured into a graph).
__global__ __launch_bounds__(256) void zero_words_kernel(int32_t* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0;
}

// Offset of row r inside a (slot, head) strip.  Blocked layouts place block r >> shift at that
// multiple of block_stride and the rows of a block row_stride apart; a plain layout is the case
// shift = 31, mask = 0x7fffffff (one block holding every row).
__device__ __forceinline__ int64_t row_offset(int r, int64_t row_stride, int64_t block_stride,
                                              int shift, int mask) {
  return (int64_t)(r >> shift) * block_stride + (int64_t)(r & mask) * row_stride;
}

// Head column `col` of pass `pass` of kv head g in group b: with (t, i) = divmod(pass * heads_per_pass
// + col, G) it is query head g*G + i of token row b*T + t.  (T = 1: the group is one sequence and
// the columns are the G heads of the kv head.)
struct Column {
  int64_t token_row;
  int head;
};
__device__ __forceinline__ Column column_of(const AttnArgs& a, int b, int g, int pass, int col) {
  const int cig = pass * a.heads_per_pass + col;
  int t = 0, i = cig;
  if (a.tokens > 1) {
    t = cig / a.real_group;
    i = cig - t * a.real_group;
  }
  return Column{(int64_t)b * a.tokens + t, g * a.real_group + i};
}
// Index of a column's (token row, head) pair in the [B, H] arrays of the workspace.
__device__ __forceinline__ int64_t column_index(const AttnArgs& a, int b, int g, int pass, int col) {
  const Column x = column_of(a, b, g, pass, col);
  return x.token_row * a.n_q_heads + x.head;
}

// One unit of work: (sequence, kv head, head pass, chunk).  The chunk index
// varies fastest so that the chunks of one strip are in flight together.
struct Item {
  int b, g, pass, chunk;
  int h0, nh;      // first query head of this pass and how many are real
  int r0, r1;      // rows [r0, r1) of the strip; r1 <= r0 means empty
  int64_t strip;   // element offset of row 0 of (slot, kv head)
};

__device__ __forceinline__ Item decode_item(const AttnArgs& a, int item) {
  Item it;
  it.chunk = item % a.n_chunks;
  int rest = item / a.n_chunks;
  it.pass = rest % a.n_pass;
  rest /= a.n_pass;
  it.g = rest % a.n_kv_heads;
  it.b = rest / a.n_kv_heads;
  it.h0 = it.g * a.group + it.pass * a.heads_per_pass;
  const int left = a.group - it.pass * a.heads_per_pass;
  it.nh = left < a.heads_per_pass ? left : a.heads_per_pass;
  const int slot = a.slot_id[it.b];
  int n = a.ctx_len[it.b] + a.ctx_bias;
  if (a.ctx_bias && (n <= 0 || n > a.row_limit)) n = 0;   // a position out of range: skipped
  n = n < a.row_limit ? n : a.row_limit;
  if (slot < 0 || slot >= a.n_slots) n = 0;
  it.r0 = it.chunk * a.chunk_rows;
  const int end = it.r0 + a.chunk_rows;
  it.r1 = n < end ? n : end;
  it.strip = (int64_t)(slot < 0 || slot >= a.n_slots ? 0 : slot) * a.slot_stride +
             (int64_t)it.g * a.head_stride;
  return it;
}

__device__ __forceinline__ int64_t partial_index(const AttnArgs& a, const Item& it, int head) {
  return ((int64_t)it.b * a.n_q_heads + head) * a.n_chunks + it.chunk;
}

// 16-byte load of K/V data that is read once per step: the non-temporal hint keeps the stream
// from displacing other lines in the caches (measured: 5.7 -> 6.1 TB/s on the large workloads).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
__device__ __forceinline__ u32x4_t stream_load(const uint16_t* p) {
  return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(p));
}

// The same from a wave-uniform base address plus a 32-bit lane offset in bytes.
// NT = false: an ordinary cached load, for rows that other waves are about to ask for as well.
template <bool NT>
__device__ __forceinline__ u32x4_t stream_load_at(const char* base, uint32_t off) {
  if constexpr (NT)
    return __builtin_nontemporal_load(reinterpret_cast<const u32x4_t*>(base + off));
  else
    return *reinterpret_cast<const u32x4_t*>(base + off);
}

// 2^x on the transcendental unit; 2^(-inf) = 0.
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }

// Two packed 16-bit values -> two floats.
template <bool BF16>
__device__ __forceinline__ void unpack2(uint32_t w, float& lo, float& hi) {
  if constexpr (BF16) {
    lo = __uint_as_float(w << 16);
    hi = __uint_as_float(w & 0xffff0000u);
  } else {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 v = __builtin_bit_cast(h2, w);
    lo = (float)v.x;
    hi = (float)v.y;
  }
}

template <bool BF16>
__device__ __forceinline__ void unpack8(const uint4& w, float (&f)[8]) {
  unpack2<BF16>(w.x, f[0], f[1]);
  unpack2<BF16>(w.y, f[2], f[3]);
  unpack2<BF16>(w.z, f[4], f[5]);
  unpack2<BF16>(w.w, f[6], f[7]);
}

// Sum over the 16 lanes of a DPP row; every lane of the row gets the total.
__device__ __forceinline__ float row16_sum(float x) {
  int v;
  v = __builtin_amdgcn_update_dpp(0, __float_as_int(x), 0xB1, 0xf, 0xf, false);   // quad_perm [1,0,3,2]
  x += __int_as_float(v);
  v = __builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x4E, 0xf, 0xf, false);   // quad_perm [2,3,0,1]
  x += __int_as_float(v);
  v = __builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x141, 0xf, 0xf, false);  // row_half_mirror
  x += __int_as_float(v);
  v = __builtin_amdgcn_update_dpp(0, __float_as_int(x), 0x140, 0xf, 0xf, false);  // row_mirror
  x += __int_as_float(v);
  return x;
}

// Maximum / sum over the four lanes hn, hn + 16, hn + 32, hn + 48 (one per 16-lane row), delivered
// to all four.  The swap instructions trade whole rows between two registers in one vector
// operation (no trip through the LDS crossbar): permlane16_swap exchanges the odd rows of its first
// operand with the even rows of its second, permlane32_swap the upper half of the first with the
// lower half of the second; fed the same value twice they return (x of the even row, x of the odd
// row) resp. (x of the lower half, x of the upper half) in every lane.
typedef uint32_t u32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ float rows_max(float x) {
  u32x2_t r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return fmaxf(__uint_as_float(r[0]), __uint_as_float(r[1]));
}
__device__ __forceinline__ float rows_sum(float x) {
  u32x2_t r = __builtin_amdgcn_permlane16_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  x = __uint_as_float(r[0]) + __uint_as_float(r[1]);
  r = __builtin_amdgcn_permlane32_swap(__float_as_uint(x), __float_as_uint(x), false, false);
  return __uint_as_float(r[0]) + __uint_as_float(r[1]);
}

// How far a column's running maximum may outgrow the exponent its sums are scaled by before they
// are rescaled (base-2 exponent: weights stay below 2^8).
constexpr float kLazyExponent = 8.f;

// Exchange with the lane 16 / 32 positions away (across the four 16-lane rows of a wave).
__device__ __forceinline__ float xor16(float x) { return __shfl_xor(x, 16, 64); }
__device__ __forceinline__ float xor32(float x) { return __shfl_xor(x, 32, 64); }

}  // namespace gh

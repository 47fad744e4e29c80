// Split-context decode attention on the matrix cores (v_mfma_f32_16x16x32).
//
// One wave owns one (sequence, kv head, head pass, chunk) and walks it in
// tiles of 32 rows.  No LDS and no barrier: both operands are loaded from
// global memory straight into the register layout the MFMA wants.  (The one
// exception -- head groups or token groups of more than 32 head columns, which
// are bound by arithmetic and not by the stream -- is the cooperative form of
// the balanced kernel: process_tile_lds below.)
//
// Lane numbering: hn = lane % 16, c = lane / 16.
//
//   scores  S^T[row][head] = sum_d K[row][d] * Q[head][d]
//     A = K tile (16 rows x 32 d), lane (hn, c) holds 8 consecutive d of row
//         rho(T, hn) for d-chunk 4*kk + c;  B = Q^T, lane (hn, c) holds the
//         same d-chunk of head hn.  Four kk steps cover d = 128, two sub-tiles
//         T cover 32 rows.  The result register i of lane (hn, c) is the score
//         of head hn against row 16T + 4i + c of the tile (rho is chosen so).
//         Loading that layout directly would touch 16 rows x 64 bytes per
//         instruction, i.e. half cache lines, which streams ~13% slower than
//         whole lines on this chip.  So a load fetches 8 rows x 128 bytes
//         instead (lanes hn >= 8 hold the second 64 bytes of row hn - 8), and
//         two DPP moves per register (rotate by 8 lanes within a 16-lane row)
//         rebuild the operand layout.
//   output  O^T[col][head] = sum_row V[row][col] * P[head][row]
//     B = P^T: lane (hn, c) needs, for its 8 contraction slots e = 4T + i,
//         P[head hn][row 16T + 4i + c] -- exactly the scores it already holds.
//     A = V^T: lane (hn, c) loads 16 bytes (columns 8hn .. 8hn+7) of those
//         same 8 rows, so that one wave-wide load reads 4 consecutive rows
//         (1 KiB contiguous); an in-register 8x8 transpose of 16-bit values
//         (v_perm_b32) turns them into the operand of column tile t, which
//         stands for columns 8*hn + t.  Result register i of lane (hn, c) in
//         tile t is column 32c + 8i + t of head hn.
//   So a lane's softmax state (running max m, partial sum l) and its 32 output
//   columns all belong to one head, and rescaling needs no cross-lane traffic
//   beyond the maximum over the four lanes of a head.
//
// The probabilities are split as p = hi + lo (both in the 16-bit type) and
// multiplied in two MFMAs, so that rounding p to 8 or 11 bits of mantissa does
// not reach the output; K.Q products are exact in fp32.
#pragma once
#include "gh_common.hpp"

namespace gh {

typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

template <bool BF16>
__device__ __forceinline__ f32x4 mfma(const u32x4& a, const u32x4& b, const f32x4& c) {
  if constexpr (BF16)
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a),
                                                   __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  else
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a),
                                                  __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
}

// Two fp32 probabilities -> packed 16-bit pair (x low, y high), round to nearest even.
template <bool BF16>
__device__ __forceinline__ uint32_t pack2(float x, float y) {
  if constexpr (BF16) {
    typedef __bf16 b2 __attribute__((ext_vector_type(2)));
    b2 v = {(__bf16)x, (__bf16)y};
    return __builtin_bit_cast(uint32_t, v);
  } else {
    typedef _Float16 h2 __attribute__((ext_vector_type(2)));
    h2 v = {(_Float16)x, (_Float16)y};
    return __builtin_bit_cast(uint32_t, v);
  }
}

// K and V registers of one 32-row tile, as loaded.
struct TileRegs {
  u32x4 k[2][2][2];  // [sub-tile T][128-byte half of the row][rows 0-7 / 8-15 of the sub-tile]
  u32x4 v[8];        // [contraction slot e = 4T + i]
};

// Lanes 8-15 of every 16-lane row take `other` rotated by 8 lanes, lanes 0-7 keep `keep`.
__device__ __forceinline__ u32x4 upper_from_rotated(const u32x4& keep, const u32x4& other) {
  u32x4 r;
#pragma unroll
  for (int w = 0; w < 4; ++w)
    r[w] = (uint32_t)__builtin_amdgcn_update_dpp((int)keep[w], (int)other[w], 0x128 /*row_ror:8*/,
                                                 0xf, 0xc, false);
  return r;
}
// Lanes 0-7 of every 16-lane row take `other` rotated by 8 lanes, lanes 8-15 keep `keep`.
__device__ __forceinline__ u32x4 lower_from_rotated(const u32x4& keep, const u32x4& other) {
  u32x4 r;
#pragma unroll
  for (int w = 0; w < 4; ++w)
    r[w] = (uint32_t)__builtin_amdgcn_update_dpp((int)keep[w], (int)other[w], 0x128 /*row_ror:8*/,
                                                 0xf, 0x3, false);
  return r;
}

// What a lane contributes to the addresses of a tile's loads: its row inside the tile (plus a
// per-register constant) and its byte column, for K and for V.
struct LaneGeom {
  int krow, vrow;          // K: register (T, ab) holds in-tile row krow + 16 T + 2 ab;  V: register e holds
                           // in-tile row vrow + 16 (e >> 2) + 4 (e & 3)
  uint32_t kcol, vcol;     // byte offsets inside the row (K: first 128-byte half)
};
__device__ __forceinline__ LaneGeom lane_geom(int hn, int c) {
  // K row rho(T, m) = 16 T + 4 (m & 3) + (m >> 2) with m = (hn & 7) + 8 ab
  return LaneGeom{4 * (hn & 3) + ((hn & 7) >> 2), c, (uint32_t)(64 * (hn >> 3) + 16 * c),
                  (uint32_t)(16 * hn)};
}

// Loads one tile.  kt / vt: address of the tile's first row in the K and the V strip, the same for
// every lane (a tile is 32-row aligned and never straddles two blocks of a blocked layout), so an
// address is that scalar plus a 32-bit lane offset: two vector instructions per address.
// `rows` (>= 1): how many of the tile's 32 rows exist; the others load the last existing row.
template <bool NT>
__device__ __forceinline__ void load_tile(TileRegs& t, const char* kt, const char* vt,
                                          uint32_t row_bytes, int rows, const LaneGeom& lg) {
  const int top = rows - 1;
  // K: one load covers 8 rows x 128 bytes (whole cache lines): lanes hn < 8 take the first
  // 64 bytes of the half-row, lanes hn >= 8 the second 64 bytes of the same row.
#pragma unroll
  for (int T = 0; T < 2; ++T) {
#pragma unroll
    for (int ab = 0; ab < 2; ++ab) {
      int r = lg.krow + 16 * T + 2 * ab;
      r = r < top ? r : top;
      const uint32_t off = __umul24((uint32_t)r, row_bytes) + lg.kcol;
#pragma unroll
      for (int half = 0; half < 2; ++half) t.k[T][half][ab] = stream_load_at<NT>(kt, off + 128 * half);
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    int r = lg.vrow + 16 * (e >> 2) + 4 * (e & 3);
    r = r < top ? r : top;
    t.v[e] = stream_load_at<NT>(vt, __umul24((uint32_t)r, row_bytes) + lg.vcol);
  }
}

// A share of a tile: what one of the W (2 or 4) waves of a cooperating workgroup fetches of it.  The
// tile's K registers come in four pairs (T, ab) of eight whole 256-byte rows, its V registers e in
// eight groups of four whole rows; wave w takes pairs w * 4/W .. and registers w * 8/W .. .
template <int W>
struct PartRegs {
  u32x4 k[8 / W];    // [pair - first pair][128-byte half of the row]
  u32x4 v[8 / W];    // [e - first e]
};
template <bool NT, int W>
__device__ __forceinline__ void load_part(PartRegs<W>& pr, const char* kt, const char* vt,
                                          uint32_t row_bytes, int rows, const LaneGeom& lg, int w) {
  const int top = rows - 1;
#pragma unroll
  for (int j = 0; j < 4 / W; ++j) {
    const int pair = w * (4 / W) + j;
    int r = lg.krow + 16 * (pair >> 1) + 2 * (pair & 1);
    r = r < top ? r : top;
    const uint32_t off = __umul24((uint32_t)r, row_bytes) + lg.kcol;
#pragma unroll
    for (int half = 0; half < 2; ++half) pr.k[2 * j + half] = stream_load_at<NT>(kt, off + 128 * half);
  }
#pragma unroll
  for (int j = 0; j < 8 / W; ++j) {
    const int e = w * (8 / W) + j;
    int rv = lg.vrow + 16 * (e >> 2) + 4 * (e & 3);
    rv = rv < top ? rv : top;
    pr.v[j] = stream_load_at<NT>(vt, __umul24((uint32_t)rv, row_bytes) + lg.vcol);
  }
}
// The tile the waves of a workgroup put together in LDS: the 32 K rows and the 32 V rows as they lie in the
// cache, 256 bytes each, at a pitch of 272 bytes -- so that the 16 rows a 16-lane group reads at
// the same byte column fall into 16 different groups of four banks.
constexpr int kLdsPitch = 272;
struct __attribute__((aligned(16))) TileLds {
  char k[32 * kLdsPitch];
  char v[32 * kLdsPitch];
};
template <int W>
__device__ __forceinline__ void put_part(TileLds& x, const PartRegs<W>& pr, int w, const LaneGeom& lg) {
#pragma unroll
  for (int j = 0; j < 4 / W; ++j) {
    const int pair = w * (4 / W) + j;
    const int rk = lg.krow + 16 * (pair >> 1) + 2 * (pair & 1);
#pragma unroll
    for (int half = 0; half < 2; ++half)
      *reinterpret_cast<u32x4*>(x.k + rk * kLdsPitch + lg.kcol + 128 * half) = pr.k[2 * j + half];
  }
#pragma unroll
  for (int j = 0; j < 8 / W; ++j) {
    const int e = w * (8 / W) + j;
    const int rv = lg.vrow + 16 * (e >> 2) + 4 * (e & 3);
    *reinterpret_cast<u32x4*>(x.v + rv * kLdsPitch + lg.vcol) = pr.v[j];
  }
}

// The online-softmax update of one tile for P passes: from the raw scores s (register e = 4T + i of
// lane (hn, c) is head column hn against tile row 16T + 4i + c) to the probabilities as two 16-bit
// operands (hi + lo), with the running exponent m and sum l brought up to date and the accumulators
// rescaled when the exponent moved.  `lim` is the number of rows the lane's head column attends
// (rows at or beyond it are masked); columns of one tile may have different limits, and a column
// may have no row at all in a tile.
template <bool BF16, int P, int NT>
__device__ __forceinline__ void softmax_tile(const f32x4 (&s)[P][2], u32x4 (&p_hi)[P], u32x4 (&p_lo)[P],
                                             f32x4 (&acc)[P][NT], float (&m)[P], float (&l)[P],
                                             float scale_log2e, int tile_row0, const int (&lim)[P],
                                             int c) {
#pragma unroll
  for (int i = 0; i < P; ++i) {
    float tv[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) tv[e] = s[i][e >> 2][e & 3] * scale_log2e;
    // rows at or beyond the column's limit are masked (select, not multiply: what lies there may
    // be anything); a tile that every column of the wave attends in full skips the selects
    if (!__all(tile_row0 + 32 <= lim[i])) {
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const int row = tile_row0 + 16 * (e >> 2) + 4 * (e & 3) + c;
        tv[e] = row < lim[i] ? tv[e] : kNegInf;
      }
    }
    float mx = kNegInf;
#pragma unroll
    for (int e = 0; e < 8; ++e) mx = fmaxf(mx, tv[e]);
    mx = rows_max(mx);
    // m is the exponent the column's running sums are scaled by.  It follows the running maximum
    // lazily: the sums are rescaled only when the maximum has grown by more than kLazyExponent
    // since the last time, so that the weights 2^(t - m) stay below 2^kLazyExponent instead of
    // below 1 -- the same relative precision, and after the first tiles of a strip hardly any
    // tile pays for a rescale.  (m = -inf: no row seen yet; then any row moves it.)
    const bool moved = mx > m[i] + kLazyExponent;
    const float mn = moved ? mx : m[i];
    // a column that has seen no row yet keeps m = -inf; subtract 0 then, so that every exponent
    // below is -inf (weight 0) rather than inf - inf
    const float ref = mn == kNegInf ? 0.f : mn;
    const float alpha = moved ? fast_exp2(m[i] - ref) : 1.f;
    m[i] = mn;
    float sum = 0.f;
    float lo[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      tv[e] = fast_exp2(tv[e] - ref);
      sum += tv[e];
    }
    l[i] = fmaf(l[i], alpha, sum);
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const uint32_t hi = pack2<BF16>(tv[2 * w], tv[2 * w + 1]);
      float h0, h1;
      unpack2<BF16>(hi, h0, h1);
      lo[2 * w] = tv[2 * w] - h0;
      lo[2 * w + 1] = tv[2 * w + 1] - h1;
      p_hi[i][w] = hi;
      p_lo[i][w] = pack2<BF16>(lo[2 * w], lo[2 * w + 1]);
    }
    if (__any(moved)) {
#pragma unroll
      for (int tcol = 0; tcol < NT; ++tcol) acc[i][tcol] *= alpha;
    }
  }
}

// One 32-row tile for P passes of 16 head columns each (own Q operand, running state and
// accumulators per pass; the K operands and the transposed V operands are built once).
template <bool BF16, int P>
__device__ __forceinline__ void process_tile(const TileRegs& t, const u32x4 (&qop)[P][4],
                                             f32x4 (&acc)[P][8], float (&m)[P], float (&l)[P],
                                             float scale_log2e, int tile_row0, const int (&lim)[P],
                                             int c) {
  // scores of head hn against this lane's 8 rows
  f32x4 s[P][2];
#pragma unroll
  for (int T = 0; T < 2; ++T) {
#pragma unroll
    for (int i = 0; i < P; ++i) s[i][T] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int half = 0; half < 2; ++half) {
      // operand of d step kk: lane (hn, c) holds d-chunk 4kk + c of row rho(T, hn)
      const u32x4 k_even = upper_from_rotated(t.k[T][half][0], t.k[T][half][1]);   // kk = 2*half
      const u32x4 k_odd = lower_from_rotated(t.k[T][half][1], t.k[T][half][0]);    // kk = 2*half + 1
#pragma unroll
      for (int i = 0; i < P; ++i) {
        s[i][T] = mfma<BF16>(k_even, qop[i][2 * half], s[i][T]);
        s[i][T] = mfma<BF16>(k_odd, qop[i][2 * half + 1], s[i][T]);
      }
    }
  }
  u32x4 p_hi[P], p_lo[P];
  softmax_tile<BF16, P, 8>(s, p_hi, p_lo, acc, m, l, scale_log2e, tile_row0, lim, c);
  // O^T += V^T P^T, one 16-column tile at a time
#pragma unroll
  for (int tcol = 0; tcol < 8; ++tcol) {
    u32x4 vt;
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      // 16-bit halves of two rows' registers -> (row 2w, row 2w+1) pair of column tcol
      const uint32_t even = t.v[2 * w][tcol >> 1], odd = t.v[2 * w + 1][tcol >> 1];
      vt[w] = (tcol & 1) ? ((even >> 16) | (odd & 0xffff0000u)) : ((even & 0xffffu) | (odd << 16));
    }
#pragma unroll
    for (int i = 0; i < P; ++i) {
      acc[i][tcol] = mfma<BF16>(vt, p_hi[i], acc[i][tcol]);
      acc[i][tcol] = mfma<BF16>(vt, p_lo[i], acc[i][tcol]);
    }
  }
}

// The same tile taken from LDS (TileLds), operands read in the layout the matrix instruction wants:
//   K: lane (hn, c) reads the 16 bytes of d-chunk 4kk + c of row rho(T, hn) = 16T + 4(hn & 3) + (hn >> 2);
//   V^T: a transposing read -- lane j of 16-lane group c hands in the address of four consecutive
//        columns 16t + 4(j & 3) .. of row 16T + 4(j >> 2) + c, and receives column 16t + j of the
//        group's four rows 16T + 4i + c, i = 0..3: contraction slots e = 4T + i of column 16t + j.
// So here result register r of lane (hn, c) in column tile t is column 16t + 4c + r of head hn
// (acc_natural), not the layout of process_tile: the stores that follow differ (store_*_natural).
typedef short v4s __attribute__((ext_vector_type(4)));
template <bool BF16, int P>
__device__ __forceinline__ void process_tile_lds(const TileLds& x, const u32x4 (&qop)[P][4],
                                                 f32x4 (&acc)[P][8], float (&m)[P], float (&l)[P],
                                                 float scale_log2e, int tile_row0,
                                                 const int (&lim)[P], int hn, int c) {
  f32x4 s[P][2];
#pragma unroll
  for (int T = 0; T < 2; ++T) {
#pragma unroll
    for (int i = 0; i < P; ++i) s[i][T] = f32x4{0.f, 0.f, 0.f, 0.f};
    const char* row = x.k + (16 * T + 4 * (hn & 3) + (hn >> 2)) * kLdsPitch + 16 * c;
#pragma unroll
    for (int kk = 0; kk < 4; ++kk) {
      const u32x4 kop = *reinterpret_cast<const u32x4*>(row + 64 * kk);
#pragma unroll
      for (int i = 0; i < P; ++i) s[i][T] = mfma<BF16>(kop, qop[i][kk], s[i][T]);
    }
  }
  u32x4 p_hi[P], p_lo[P];
  softmax_tile<BF16, P, 8>(s, p_hi, p_lo, acc, m, l, scale_log2e, tile_row0, lim, c);
  const char* vrow = x.v + (4 * (hn >> 2) + c) * kLdsPitch + 8 * (hn & 3);
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    typedef v4s __attribute__((address_space(3))) * lds_v4s;
    const v4s lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(vrow + 32 * t));
    const v4s hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4s)(vrow + 16 * kLdsPitch + 32 * t));
    typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
    const u32x2 a = __builtin_bit_cast(u32x2, lo), b = __builtin_bit_cast(u32x2, hi);
    const u32x4 vt = {a[0], a[1], b[0], b[1]};
#pragma unroll
    for (int i = 0; i < P; ++i) {
      acc[i][t] = mfma<BF16>(vt, p_hi[i], acc[i][t]);
      acc[i][t] = mfma<BF16>(vt, p_lo[i], acc[i][t]);
    }
  }
}

// Loads the Q operand of the nh head columns of pass `pass` of kv head g in group b.  Padding lanes
// (hn >= nh) load column 0 as well -- the load is unconditional so that nothing has to wait for it
// at the point of issue -- and are zeroed by keep_real_heads() when the operand is taken into use.
__device__ __forceinline__ void load_q(u32x4 (&qop)[4], const AttnArgs& a, int b, int g, int pass,
                                       int nh, int hn, int c) {
  const Column x = column_of(a, b, g, pass, hn < nh ? hn : 0);
#pragma unroll
  for (int kk = 0; kk < 4; ++kk)
    qop[kk] = *reinterpret_cast<const u32x4*>(
        a.q + x.token_row * a.q_batch_stride + x.head * kHeadDim + 32 * kk + 8 * c);
}
__device__ __forceinline__ void keep_real_heads(u32x4 (&dst)[4], const u32x4 (&src)[4], int nh,
                                                int hn) {
#pragma unroll
  for (int kk = 0; kk < 4; ++kk) dst[kk] = hn < nh ? src[kk] : u32x4{0u, 0u, 0u, 0u};
}

// Raw buffer descriptor word 3 for 32-bit raw access on this architecture, and the cache-policy
// operand of buffer instructions: bit 0 = sc0, bit 1 = nt, bit 4 = sc1.
constexpr int kRawBufferFlags = 0x00020000;
constexpr int kWriteThrough = 0x11;

// Exchange between lanes that differ in one bit of the lane number: afterwards the lanes with
// that bit clear hold in `hi` what their partner had in `lo`, and the lanes with the bit set hold
// in `lo` what their partner had in `hi` (the other halves stay).  No selects: the data parallel
// primitives write only the enabled banks (bank = 4 lanes) or rows (row = 16 lanes).
__device__ __forceinline__ void swap_lane_bit2(f32x4& lo, f32x4& hi) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int l = __float_as_int(lo[e]), h = __float_as_int(hi[e]);
    // banks 0 and 2 (bit clear) read the lane 4 above, banks 1 and 3 the lane 4 below
    hi[e] = __int_as_float(__builtin_amdgcn_update_dpp(h, l, 0x12c /*row_ror:12*/, 0xf, 0x5, false));
    lo[e] = __int_as_float(__builtin_amdgcn_update_dpp(l, h, 0x124 /*row_ror:4*/, 0xf, 0xa, false));
  }
}
__device__ __forceinline__ void swap_lane_bit3(f32x4& lo, f32x4& hi) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const int l = __float_as_int(lo[e]), h = __float_as_int(hi[e]);
    hi[e] = __int_as_float(__builtin_amdgcn_update_dpp(h, l, 0x128 /*row_ror:8*/, 0xf, 0x3, false));
    lo[e] = __int_as_float(__builtin_amdgcn_update_dpp(l, h, 0x128 /*row_ror:8*/, 0xf, 0xc, false));
  }
}
__device__ __forceinline__ void swap_lane_bit4(f32x4& lo, f32x4& hi) {
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    // odd rows of the first operand trade places with even rows of the second
    const u32x2 r = __builtin_amdgcn_permlane16_swap(__float_as_uint(lo[e]), __float_as_uint(hi[e]),
                                                     false, false);
    lo[e] = __uint_as_float(r[0]);
    hi[e] = __uint_as_float(r[1]);
  }
}

// Writes the running state as partial record `slot` of heads h0 .. h0+nh-1 of sequence b.
//
// Record stores are the expensive part of a strip border: on a ragged batch they are 0.5% of the
// bytes and cost 10% of the kernel's time when written with plain stores (measured by leaving them
// out), because every line written interrupts the read stream in memory.  Two measures, which only
// help together (measured: 76% of peak bandwidth with either alone, 81% with both):
//  * whole lines.  Lane (hn, c) holds columns 32c .. 32c+31 of head hn as eight 16-byte chunks;
//    stored as they are, one instruction would put 16 bytes into each of 64 different cache lines.
//    Three exchange stages trade the chunk index for lane bits 2, 3 and 4 instead: afterwards lane
//    L, register r = r0 + 2 r1 + 4 r2 holds
//        head   (L & 3) + 4 r0 + 8 r1,    chunk  (L >> 2) & 7  of column block  r2 + 2 (L >> 5),
//    so the eight lanes that differ in bits 2-4 write one whole 128-byte line per instruction;
//  * write-through stores (see below).
__device__ __forceinline__ void whole_line_chunks(f32x4 (&x)[8]) {
#pragma unroll
  for (int q = 0; q < 8; q += 2) swap_lane_bit2(x[q], x[q + 1]);
#pragma unroll
  for (int q = 0; q < 8; ++q)
    if (!(q & 2)) swap_lane_bit3(x[q], x[q + 2]);
#pragma unroll
  for (int q = 0; q < 4; ++q) swap_lane_bit4(x[q], x[q + 4]);
}

__device__ __forceinline__ void store_record(const AttnArgs& a, int b, int g, int pass, int nh,
                                             int slot, const f32x4 (&acc)[8], float m, float l,
                                             int hn, int c) {
  l = rows_sum(l);                     // the four lanes of a head share m; add their partial sums
  f32x4 x[8];                          // chunk q = columns 32c + 4q .. 32c + 4q + 3
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    // register i of column tile t is column 32c + 8i + t
    x[2 * i] = f32x4{acc[0][i], acc[1][i], acc[2][i], acc[3][i]};
    x[2 * i + 1] = f32x4{acc[4][i], acc[5][i], acc[6][i], acc[7][i]};
  }
  whole_line_chunks(x);

  // Write-through stores (sc0 sc1): among the store policies this one disturbs the read stream
  // least (a streaming-read probe that writes 4 KiB per wave now and then: 7.0 TB/s without stores,
  // 6.3 with plain stores, 6.6-6.7 with write-through or non-temporal ones), and unlike the
  // non-temporal policy it leaves the records in cache for the merge kernel.  The policy bits are
  // only reachable through buffer instructions, so the record of the wave's first head becomes the
  // buffer base; its range ends with the last real column (the columns' records lie at increasing
  // addresses), and b, g, pass and slot are wave-uniform.
  const int lane = 16 * c + hn;
  const int64_t pitch = (int64_t)a.n_chunks * kHeadDim;      // floats between (token row, head) pairs
  const int64_t first = column_index(a, b, g, pass, 0);
  const int64_t last = column_index(a, b, g, pass, nh - 1);
  float* base = a.ws_o + (first * a.n_chunks + slot) * kHeadDim;
  const __amdgpu_buffer_rsrc_t rec = __builtin_amdgcn_make_buffer_rsrc(
      base, 0, (int)(((last - first) * pitch + kHeadDim) * 4), kRawBufferFlags);
  const int col = 64 * (lane >> 5) + 4 * ((lane >> 2) & 7);
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int head = (lane & 3) + 4 * k;                     // head column of registers k and k + 4
    if (head < nh) {
      const int at = (int)(((column_index(a, b, g, pass, head) - first) * pitch + col) * 4);
      __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, x[k]), rec, at, 0,
                                             kWriteThrough);
      __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, x[k + 4]), rec, at + 32 * 4,
                                             0, kWriteThrough);
    }
  }
  if (hn < nh && c == 0) {
    const int64_t pi = column_index(a, b, g, pass, hn) * a.n_chunks + slot;
    if (a.ctx_bias) {
      // one-launch step: another wave of this launch reads the record, possibly through another
      // L2; device-scope stores go through to memory like the rows above
      __hip_atomic_store(a.ws_m + pi, m, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      __hip_atomic_store(a.ws_l + pi, l, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    } else {
      a.ws_m[pi] = m;
      a.ws_l[pi] = l;
    }
  }
}

// Final result of head columns whose rows this wave covered alone: o / l (zeros for a column
// without rows), stored straight into the output -- what the merge would compute from this one
// record, bit for bit (its weight is 2^0) -- in fp32 or rounded once to the 16-bit type.
template <bool BF16>
__device__ __forceinline__ void store_final(const AttnArgs& a, int b, int g, int pass, int nh,
                                            const f32x4 (&acc)[8], float l, int hn, int c) {
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  l = rows_sum(l);
  f32x4 x[8];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    x[2 * i] = f32x4{acc[0][i], acc[1][i], acc[2][i], acc[3][i]};
    x[2 * i + 1] = f32x4{acc[4][i], acc[5][i], acc[6][i], acc[7][i]};
  }
#pragma unroll
  for (int q = 0; q < 8; ++q)
#pragma unroll
    for (int e = 0; e < 4; ++e)            // (+ 0: the merge's 1 * o + 0 turns a -0 into +0)
      x[q][e] = l > 0.f ? (x[q][e] + 0.f) / l : 0.f;
  whole_line_chunks(x);

  const int lane = 16 * c + hn;
  const bool wide = a.out_kind == 1;                         // fp32, else the 16-bit type
  const int esize = wide ? 4 : 2;
  const int64_t first = column_index(a, b, g, pass, 0);
  const int64_t last = column_index(a, b, g, pass, nh - 1);
  char* base = static_cast<char*>(a.out) + first * kHeadDim * esize;
  const __amdgpu_buffer_rsrc_t dst = __builtin_amdgcn_make_buffer_rsrc(
      base, 0, (int)((last - first + 1) * kHeadDim * esize), kRawBufferFlags);
  const int col = 64 * (lane >> 5) + 4 * ((lane >> 2) & 7);
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int head = (lane & 3) + 4 * k;
    if (head < nh) {
      const int at = (int)((column_index(a, b, g, pass, head) - first) * kHeadDim + col);
      if (wide) {
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, x[k]), dst, at * 4, 0,
                                               kWriteThrough);
        __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, x[k + 4]), dst,
                                               (at + 32) * 4, 0, kWriteThrough);
      } else {
        const u32x2 lo = {pack2<BF16>(x[k][0], x[k][1]), pack2<BF16>(x[k][2], x[k][3])};
        const u32x2 hi = {pack2<BF16>(x[k + 4][0], x[k + 4][1]), pack2<BF16>(x[k + 4][2], x[k + 4][3])};
        __builtin_amdgcn_raw_buffer_store_b64(lo, dst, at * 2, 0, kWriteThrough);
        __builtin_amdgcn_raw_buffer_store_b64(hi, dst, (at + 32) * 2, 0, kWriteThrough);
      }
    }
  }
}

// The same two stores for accumulators in the layout of process_tile_lds: register r of column tile
// t is column 16t + 4c + r, so a lane writes eight 16-byte pieces per head column and the four lanes
// of a head cover 64 bytes per instruction.  (These are the stores of launches that are bound by
// arithmetic, not by the memory stream: half lines are good enough.)
__device__ __forceinline__ void store_record_natural(const AttnArgs& a, int b, int g, int pass, int nh,
                                                     int slot, const f32x4 (&acc)[8], float m, float l,
                                                     int hn, int c) {
  l = rows_sum(l);
  const int64_t pitch = (int64_t)a.n_chunks * kHeadDim;
  const int64_t first = column_index(a, b, g, pass, 0);
  const int64_t last = column_index(a, b, g, pass, nh - 1);
  float* base = a.ws_o + (first * a.n_chunks + slot) * kHeadDim;
  const __amdgpu_buffer_rsrc_t rec = __builtin_amdgcn_make_buffer_rsrc(
      base, 0, (int)(((last - first) * pitch + kHeadDim) * 4), kRawBufferFlags);
  if (hn < nh) {
    const int64_t mine = column_index(a, b, g, pass, hn);
    const int at = (int)(((mine - first) * pitch + 4 * c) * 4);
#pragma unroll
    for (int t = 0; t < 8; ++t)
      __builtin_amdgcn_raw_buffer_store_b128(__builtin_bit_cast(u32x4, acc[t]), rec, at + 64 * t, 0,
                                             kWriteThrough);
    if (c == 0) {
      a.ws_m[mine * a.n_chunks + slot] = m;
      a.ws_l[mine * a.n_chunks + slot] = l;
    }
  }
}
template <bool BF16>
__device__ __forceinline__ void store_final_natural(const AttnArgs& a, int b, int g, int pass, int nh,
                                                    const f32x4 (&acc)[8], float l, int hn, int c) {
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  l = rows_sum(l);
  if (hn >= nh) return;
  const int64_t at = column_index(a, b, g, pass, hn) * kHeadDim + 4 * c;
#pragma unroll
  for (int t = 0; t < 8; ++t) {
    f32x4 x;
#pragma unroll
    for (int e = 0; e < 4; ++e)            // (+ 0: the merge's 1 * o + 0 turns a -0 into +0)
      x[e] = l > 0.f ? (acc[t][e] + 0.f) / l : 0.f;
    if (a.out_kind == 1) {
      *reinterpret_cast<f32x4*>(static_cast<float*>(a.out) + at + 16 * t) = x;
    } else {
      const u32x2 w = {pack2<BF16>(x[0], x[1]), pack2<BF16>(x[2], x[3])};
      *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(a.out) + at + 16 * t) = w;
    }
  }
}

// The append of the one-launch step.  There the row a step appends is a tile of its own at the end
// of the strip, loaded from k_new / v_new like any tile with a single row (every lane's row clamps
// to it).  The lanes whose registers stand for in-tile row `top` (0 for that tile; not one of the
// clamped copies) write the row to its place in the caches.  krow / vrow: address of that row in
// the K and the V strip.  A bit copy of what was loaded.
__device__ __forceinline__ void store_new_row(const TileRegs& t, char* krow, char* vrow, int top,
                                              const LaneGeom& lg) {
#pragma unroll
  for (int T = 0; T < 2; ++T) {
#pragma unroll
    for (int ab = 0; ab < 2; ++ab) {
      if (lg.krow + 16 * T + 2 * ab == top) {
#pragma unroll
        for (int half = 0; half < 2; ++half)
          *reinterpret_cast<u32x4*>(krow + lg.kcol + 128 * half) = t.k[T][half][ab];
      }
    }
  }
#pragma unroll
  for (int e = 0; e < 8; ++e) {
    if (lg.vrow + 16 * (e >> 2) + 4 * (e & 3) == top)
      *reinterpret_cast<u32x4*>(vrow + lg.vcol) = t.v[e];
  }
}

// Merge of the first n_rec partial records of the nh head columns of one pass (the rule of
// decode_reduce_kernel), by one wave, for all columns at once: lanes 0-31 take the even columns,
// lanes 32-63 the odd ones, four output columns each.  NJ = column pairs (4 for up to 8 columns, 8
// for up to 16), R = records per batch: the records are read R at a time -- all loads of a batch in
// flight together, one memory round trip -- and folded into running (exponent, sum, row) triples.
// The order of the arithmetic is fixed by the record index alone.
// An address that is the same in every lane, moved to scalar registers.
__device__ __forceinline__ float* uniform_address(float* p) {
  const uint64_t v = reinterpret_cast<uint64_t>(p);
  const uint32_t lo = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)v);
  const uint32_t hi = (uint32_t)__builtin_amdgcn_readfirstlane((int)(uint32_t)(v >> 32));
  return reinterpret_cast<float*>(((uint64_t)hi << 32) | lo);
}

template <bool BF16, int NJ, int R>
__device__ __forceinline__ void merge_columns(const AttnArgs& a, int b, int g, int pass, int nh,
                                              int n_rec, int lane) {
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  const int half = lane >> 5, cg = lane & 31;
  // The records were written by other waves of this launch, with write-through stores: they are
  // loaded at device scope, past the caches that are not kept coherent between the chip's L2
  // slices.  (Buffer loads carry that policy; the records of the pass's columns lie at increasing
  // addresses from the first column's, within 2 GiB -- the launch checks that.)
  // (b, g and pass are the same in every lane; say so, or each load becomes a loop over lanes)
  const int64_t first = column_index(a, __builtin_amdgcn_readfirstlane(b), __builtin_amdgcn_readfirstlane(g),
                                     __builtin_amdgcn_readfirstlane(pass), 0);
  const __amdgpu_buffer_rsrc_t rec = __builtin_amdgcn_make_buffer_rsrc(
      uniform_address(a.ws_o + first * a.n_chunks * kHeadDim), 0, 0x7fffffff, kRawBufferFlags);
  const __amdgpu_buffer_rsrc_t rec_m = __builtin_amdgcn_make_buffer_rsrc(
      uniform_address(a.ws_m + first * a.n_chunks), 0, 0x7fffffff, kRawBufferFlags);
  const __amdgpu_buffer_rsrc_t rec_l = __builtin_amdgcn_make_buffer_rsrc(
      uniform_address(a.ws_l + first * a.n_chunks), 0, 0x7fffffff, kRawBufferFlags);
  float M[NJ], L[NJ];
  f32x4 acc[NJ];
  int rel[NJ];                                                   // first record of the column, from `first`
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    const int hc = 2 * j + half;
    // padding lanes shadow column 0
    rel[j] = (int)((column_index(a, b, g, pass, hc < nh ? hc : 0) - first) * a.n_chunks);
    M[j] = kNegInf;
    L[j] = 0.f;
    acc[j] = f32x4{0.f, 0.f, 0.f, 0.f};
  }
  for (int r0 = 0; r0 < n_rec; r0 += R) {
    float mm[NJ][R], ll[NJ][R];
    f32x4 oo[NJ][R];
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
#pragma unroll
      for (int u = 0; u < R; ++u) {
        const int r = r0 + u < n_rec ? r0 + u : n_rec - 1;       // past the end: the last one again, weight 0
        const int at = rel[j] + r;
        mm[j][u] = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rec_m, at * 4, 0, kWriteThrough));
        const float lr = __builtin_bit_cast(float, __builtin_amdgcn_raw_buffer_load_b32(rec_l, at * 4, 0, kWriteThrough));
        ll[j][u] = r0 + u < n_rec ? lr : 0.f;
        oo[j][u] = __builtin_bit_cast(f32x4, __builtin_amdgcn_raw_buffer_load_b128(
            rec, (at * kHeadDim + 4 * cg) * 4, 0, kWriteThrough));
      }
    }
#pragma unroll
    for (int j = 0; j < NJ; ++j) {
      float mx = M[j];
#pragma unroll
      for (int u = 0; u < R; ++u) {
        mm[j][u] = ll[j][u] > 0.f ? mm[j][u] : kNegInf;          // a record without rows carries no exponent
        mx = fmaxf(mx, mm[j][u]);
      }
      if (mx != kNegInf) {
        const float keep = fast_exp2(M[j] - mx);                 // 0 while nothing has been folded in
        f32x4 x = acc[j] * keep;
        float sum = L[j] * keep;
#pragma unroll
        for (int u = 0; u < R; ++u) {
          const float w = fast_exp2(mm[j][u] - mx);
          if (w > 0.f) {                                         // an empty record's row is unspecified
#pragma unroll
            for (int e = 0; e < 4; ++e) x[e] = fmaf(w, oo[j][u][e], x[e]);
          }
          sum = fmaf(w, ll[j][u], sum);
        }
        acc[j] = x;
        L[j] = sum;
        M[j] = mx;
      }
    }
  }
#pragma unroll
  for (int j = 0; j < NJ; ++j) {
    if (2 * j + half < nh) {
      const int64_t row = first + rel[j] / a.n_chunks;
      f32x4 x;
#pragma unroll
      for (int e = 0; e < 4; ++e) x[e] = L[j] > 0.f ? acc[j][e] / L[j] : 0.f;
      if (a.out_kind == 1) {
        *reinterpret_cast<f32x4*>(static_cast<float*>(a.out) + row * kHeadDim + 4 * cg) = x;
      } else {
        const u32x2 w = {pack2<BF16>(x[0], x[1]), pack2<BF16>(x[2], x[3])};
        *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(a.out) + row * kHeadDim + 4 * cg) = w;
      }
    }
  }
}

// Rows [r0, r1) (r0 < r1) of one strip for the heads h0 .. h0+nh-1 of sequence b, written as
// partial record `slot` of those heads.
template <bool BF16>
__device__ __forceinline__ void run_strip(const AttnArgs& a, int b, int g, int pass, int nh,
                                          int64_t strip, int r0, int r1, int slot, int lane) {
  const int hn = lane & 15, c = lane >> 4;

  // Q operand: d-chunk 4kk + c of head hn (zeros for the padding heads).
  u32x4 qraw[4], qop[1][4];
  load_q(qraw, a, b, g, pass, nh, hn, c);
  keep_real_heads(qop[0], qraw, nh, hn);

  f32x4 acc[1][8];
#pragma unroll
  for (int tcol = 0; tcol < 8; ++tcol) acc[0][tcol] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m[1] = {kNegInf}, l[1] = {0.f};
  const int lim[1] = {r1};

  const LaneGeom lg = lane_geom(hn, c);
  const uint32_t row_bytes = (uint32_t)a.row_stride * 2u;
  const int last = r1 - 1;
  // tile at row0 (a multiple of 32); past the end, the tile that holds the last row once more
  auto issue = [&](TileRegs& t, int row0) {
    row0 = row0 <= last ? row0 : last & ~31;
    const int64_t at = strip + row_offset(row0, a.row_stride, a.block_stride, a.block_shift, a.block_mask);
    load_tile<true>(t, reinterpret_cast<const char*>(a.k_cache + at),
                    reinterpret_cast<const char*>(a.v_cache + at), row_bytes, r1 - row0, lg);
  };

  // Two register tiles in flight.  The loads are issued unconditionally (rows past the end are
  // clamped to the last row, whose lines are already in cache) so that the number of outstanding
  // loads is known at every wait and a tile's arithmetic overlaps the next tile's loads.
  TileRegs ta, tb;
  issue(ta, r0);
  for (int row0 = r0; row0 < r1; row0 += 64) {
    issue(tb, row0 + 32);
    process_tile<BF16, 1>(ta, qop, acc, m, l, a.scale_log2e, row0, lim, c);
    issue(ta, row0 + 64);
    if (row0 + 32 < r1) process_tile<BF16, 1>(tb, qop, acc, m, l, a.scale_log2e, row0 + 32, lim, c);
  }

  store_record(a, b, g, pass, nh, slot, acc[0], m[0], l[0], hn, c);
}

// Marks partial records [slot0, slot1) of heads h0 .. h0+nh-1 of sequence b as empty.
__device__ __forceinline__ void mark_empty(const AttnArgs& a, int b, int h0, int nh, int slot0,
                                           int slot1, int lane) {
  const int n = slot1 - slot0;
  for (int idx = lane; idx < nh * n; idx += 64) {
    const int64_t pi = ((int64_t)b * a.n_q_heads + h0 + idx / n) * a.n_chunks + slot0 + idx % n;
    a.ws_m[pi] = kNegInf;
    a.ws_l[pi] = 0.f;
  }
}

// Fixed split: one wave per (sequence, kv head, head pass, chunk of chunk_rows rows).
template <bool BF16>
__global__ __launch_bounds__(64, 2) void attn_mfma_kernel(const AttnArgs a) {
  const Item it = decode_item(a, blockIdx.x);
  const int lane = threadIdx.x;
  if (it.chunk == 0 && lane < it.nh)            // every record of a head is written in this split
    a.ws_n[(int64_t)it.b * a.n_q_heads + it.h0 + lane] = a.n_chunks;
  if (it.r1 <= it.r0) {
    mark_empty(a, it.b, it.h0, it.nh, it.chunk, it.chunk + 1, lane);
    return;
  }
  run_strip<BF16>(a, it.b, it.g, it.pass, it.nh, it.strip, it.r0, it.r1, it.chunk, lane);
}

// Balanced split.  All strips (sequence, kv head, head pass) are laid end to end in units of
// 32-row tiles (a strip without rows counts as one tile) and the total is cut into equal shares,
// one per wave, so that every wave streams the same number of bytes however ragged the batch is.
// A share that crosses strip borders yields one partial record per strip it touches; the record
// index within a strip is the wave's distance from the first wave that touched that strip.  The
// wave that finishes a strip writes the number of records the strip's heads use.
//
// A wave walks its share as one continuous stream of tiles: the loads of the next tile are in
// flight while a tile is computed, across strip borders too, and the Q operand of the following
// strip is fetched one strip ahead.  (Draining the stream at every strip border cost about 20 us
// per border under load -- three dependent memory round trips.)
//
// A group is T consecutive token rows of the batch that address one slot (T = 1: one sequence).
// Its strips stream the rows the longest of its tokens attends; each head column of a tile belongs
// to one token and is masked at that token's own length, so the K/V rows of a prefill chunk are
// read once for T tokens.  Token rows that are empty, invalid or on another slot than the group's
// first live row get no rows (their output is zero).
//
// Dynamic LDS, three arrays indexed by group: cum[B + 1] = tiles of all strips of earlier groups
// (all strips of a group have the same number of tiles), rows[B] = rows streamed (0 for a group
// without a live token), base[B] = slot id (0 for such a group).
struct TileCursor {
  uint32_t t;       // global tile index
  int b;            // sequence
  uint32_t sib;     // strip within the sequence: kv head * n_pass + pass
  uint32_t lt;      // tile within the strip
  uint32_t tiles;   // tiles per strip of this sequence (>= 1)
  int n;            // rows attended of this sequence
  int slot;         // cache slot (0 when n == 0)
  // kept for the cursors that address tiles (not for the one that runs ahead for Q rows):
  int g;            // kv head of the strip
  int64_t strip;    // element offset of the strip's row 0 in the caches
  int64_t off;      // element offset of the tile's first row inside the strip
};

//
// P = passes of 16 head columns a wave carries through a strip at once (own Q operand, running
// state and accumulators per pass, one stream of tiles for all): 1 for decode, 2 for token groups
// with more than 16 head columns, at one wave per SIMD instead of two.
// COOP: 0, or the number of waves (2 or 4) of a workgroup that is one worker: its waves walk the
//       same tiles, each with its own P passes, fetch a share of every tile each, put the tile
//       together in LDS and read their operands from there.
// FUSED: the whole step in one launch (see AttnArgs): append, attention and merge.
template <bool BF16, bool GROUPED, int P, int COOP, bool FUSED>
__global__ __launch_bounds__(COOP ? 64 * COOP : 256, COOP ? 2 : 1)
void attn_mfma_balanced_kernel(const AttnArgs a) {
  static_assert(!(FUSED && GROUPED), "the one-launch step is for batches of one token per slot");
  static_assert(!(FUSED && COOP), "the one-launch step runs a wave per worker");
  constexpr int kThreads = COOP ? 64 * COOP : 256;
  extern __shared__ uint32_t lds[];
  __shared__ uint32_t part[kThreads / 64];
  const int tid = threadIdx.x;
  const int B = a.batch;
  uint32_t* cum = lds;                                        // [B + 1]
  int* rows = reinterpret_cast<int*>(lds + B + 1);            // [B]
  int* slots = rows + B;                                      // [B]
  const uint32_t spb = (uint32_t)(a.n_kv_heads * a.n_pass);   // strips per sequence

  for (int b = tid; b < B; b += kThreads) {
    int slot = 0, n = 0;
    for (int t = 0; t < a.tokens; ++t) {
      const int st = a.slot_id[(int64_t)b * a.tokens + t];
      int nt = a.ctx_len[(int64_t)b * a.tokens + t];
      if constexpr (FUSED) {
        // ctx_len[] holds the position of the new row: it must lie inside the slot and inside the
        // declared bound, else the sequence is skipped (no append, result zero) and flagged
        const bool bad_slot = st < 0 || st >= a.n_slots, bad_pos = nt < 0 || nt >= a.row_limit;
        if ((bad_slot || bad_pos) && a.dev_status && blockIdx.x == 0)
          atomicOr(a.dev_status, (bad_slot ? 1 : 0) | (bad_pos ? 2 : 0));
        nt = bad_pos ? 0 : nt + 1;
      } else if (a.ctx_bias) {
        // positions again, but the rows are appended already (the step as three kernels): a
        // position out of range was skipped by the append and attends nothing
        nt = nt < 0 || nt >= a.row_limit ? 0 : nt + 1;
      }
      nt = nt < a.row_limit ? nt : a.row_limit;
      if (st < 0 || st >= a.n_slots || nt <= 0) continue;
      if (n == 0) slot = st;                     // the first live token row names the group's slot
      if (st == slot) n = nt > n ? nt : n;
    }
    rows[b] = n;
    slots[b] = slot;
    // (one-launch step: the cached rows 0 .. n-2 in tiles, then the new row as a tile of its own)
    cum[b + 1] = (n > 0 ? ((uint32_t)(n - (FUSED ? 1 : 0) + 31) >> 5) + (FUSED ? 1u : 0u) : 1u) * spb;
  }
  if (tid == 0) cum[0] = 0;
  __syncthreads();
  const int per = (B + kThreads - 1) / kThreads;
  const int lo = tid * per, hi = lo + per < B ? lo + per : B;
  uint32_t sum = 0;
  for (int b = lo; b < hi; ++b) sum += cum[b + 1];
  // prefix over the threads' sums: inside each wave by lane shuffles, across the waves through
  // one LDS word per wave (one barrier instead of two per doubling step)
  uint32_t upto = sum;                         // inclusive, within the wave
#pragma unroll
  for (int off = 1; off < 64; off <<= 1) {
    const uint32_t below = __shfl_up(upto, off, 64);
    if ((tid & 63) >= off) upto += below;
  }
  if ((tid & 63) == 63) part[tid >> 6] = upto;
  __syncthreads();
  uint32_t run = upto - sum;                   // exclusive prefix of this thread's segment
  for (int w = 0; w < (tid >> 6); ++w) run += part[w];
  for (int b = lo; b < hi; ++b) {
    run += cum[b + 1];
    cum[b + 1] = run;
  }
  __syncthreads();

  // Everything below is the same for all lanes of a wave: keep it in scalar registers.
  auto uni = [](uint32_t x) { return (uint32_t)__builtin_amdgcn_readfirstlane((int)x); };
  const uint32_t total = uni(cum[B]);
  const int lane = tid & 63;
  const int hn = lane & 15, c = lane >> 4;
  // Worker: one wave, or (COOP) the waves of the workgroup, which walk the same tiles, each
  // with its own passes; gw numbers the workers.
  const uint32_t wave = uni(tid >> 6);
  constexpr uint32_t n_share = COOP ? (uint32_t)COOP : 1u;
  const uint32_t gw = COOP ? blockIdx.x : blockIdx.x * 4 + wave;
  const int wsub = COOP ? (int)wave * P : 0;                   // first pass of this wave in a strip's set
  uint32_t share = (total + a.n_workers - 1) / a.n_workers;    // tiles per worker
  share = share > (uint32_t)a.min_share ? share : (uint32_t)a.min_share;
  const uint32_t t0 = gw * share;
  const uint32_t t_end = t0 + share < total ? t0 + share : total;
  if (t0 >= total) return;

  auto enter_sequence = [&](TileCursor& cu) {
    const uint32_t cb = uni(cum[cu.b]);
    cu.tiles = (uni(cum[cu.b + 1]) - cb) / spb;
    cu.n = (int)uni((uint32_t)rows[cu.b]);
    cu.slot = (int)uni((uint32_t)slots[cu.b]);
  };
  // The address of a tile is kept up to date step by step (a few scalar additions per tile; worked
  // out from scratch it is a division and five 64-bit products).
  const int64_t tile_step = 32 * a.row_stride;
  const int64_t block_jump = a.block_stride - ((int64_t)a.block_mask + 1) * a.row_stride;
  auto enter_strip = [&](TileCursor& cu) {                     // cu.lt is 0
    cu.g = (int)(cu.sib / (uint32_t)a.n_pass);
    cu.strip = (int64_t)cu.slot * a.slot_stride + (int64_t)cu.g * a.head_stride;
    cu.off = 0;
  };
  auto advance = [&](TileCursor& cu) {                         // caller keeps cu.t + 1 < total
    ++cu.t;
    if (++cu.lt == cu.tiles) {
      cu.lt = 0;
      if (++cu.sib == spb) {
        cu.sib = 0;
        ++cu.b;
        enter_sequence(cu);
      }
      enter_strip(cu);
    } else {
      cu.off += tile_step;
      // (a blocked layout: the first tile of the next block; a plain one has a single block)
      if (((cu.lt << 5) & (uint32_t)a.block_mask) == 0) cu.off += block_jump;
    }
  };
  // Strip `sib` of a group: kv head g, passes pass0 .. pass0 + P - 1 of which nh[i] columns are
  // real (0 for a pass beyond the group's columns; the first pass of a strip always has some).
  auto pass_of = [&](uint32_t sib, int& g, int& pass0, int (&nh)[P]) {
    g = (int)(sib / (uint32_t)a.n_pass);
    pass0 = (int)(sib % (uint32_t)a.n_pass) * (P * (int)n_share) + wsub;
#pragma unroll
    for (int i = 0; i < P; ++i) {
      const int left = a.group - (pass0 + i) * a.heads_per_pass;
      nh[i] = left < 0 ? 0 : left < a.heads_per_pass ? left : a.heads_per_pass;
    }
  };
  // Rows the lane's head column attends.  GROUPED (T > 1): the token row's own length if it is live
  // and on the group's slot, loaded with the Q operand, unconditionally, and taken into use with
  // it.  Otherwise it is the length of the strip's sequence, which the cursor already holds.
  struct Limit { int slot, n; };
  auto load_limit = [&](const TileCursor& cu, int b, int g, int pass, int nh) {
    if constexpr (GROUPED) {
      const int64_t row = column_of(a, b, g, pass, hn < nh ? hn : 0).token_row;
      return Limit{a.slot_id[row], a.ctx_len[row]};
    } else {
      return Limit{cu.slot, cu.n};
    }
  };
  auto rows_of = [&](const Limit& x, int slot) {
    if constexpr (GROUPED) {
      const int n = x.n < a.row_limit ? x.n : a.row_limit;
      return x.slot == slot && n > 0 ? n : 0;
    } else {
      return x.n;
    }
  };
  const LaneGeom lg = lane_geom(hn, c);
  const uint32_t row_bytes = (uint32_t)a.row_stride * 2u;
  // Where the tile under a cursor is read from, and how many of its 32 rows exist.
  auto tile_source = [&](const TileCursor& cu, const char*& kt, const char*& vt, int& rows) {
    const int g = cu.g;
    const int row0 = (int)cu.lt * 32;
    // A strip without rows reads the first 256 bytes of q instead: the loads stay unconditional,
    // and no cache address is touched that the caller did not declare attended (a paged cache
    // may have nothing mapped there).
    kt = reinterpret_cast<const char*>(a.q);
    vt = kt;
    rows = 1;
    if (cu.n > 0) {
      const int64_t at = cu.strip + cu.off;
      kt = reinterpret_cast<const char*>(a.k_cache + at);
      vt = reinterpret_cast<const char*>(a.v_cache + at);
      rows = cu.n - row0;
      if constexpr (FUSED) {
        rows = cu.n - 1 - row0;                                // the cache holds rows 0 .. n-2
        if (cu.lt + 1 == cu.tiles) {                           // the last tile is the new row alone
          const int64_t from = (int64_t)cu.b * a.new_batch_stride + (int64_t)g * kHeadDim;
          kt = reinterpret_cast<const char*>(a.k_new + from);
          vt = reinterpret_cast<const char*>(a.v_new + from);
          rows = 1;
        }
      }
    }
  };
  // (every row is read once, by one wave: keep the stream out of the caches' way)
  auto issue = [&](TileRegs& regs, const TileCursor& cu) {
    const char *kt, *vt;
    int rows;
    tile_source(cu, kt, vt, rows);
    load_tile<true>(regs, kt, vt, row_bytes, rows, lg);
  };
  constexpr int kPartWaves = COOP ? COOP : 4;
  auto issue_part = [&](PartRegs<kPartWaves>& pr, const TileCursor& cu) {
    const char *kt, *vt;
    int rows;
    tile_source(cu, kt, vt, rows);
    load_part<true, kPartWaves>(pr, kt, vt, row_bytes, rows, lg, (int)wave);
  };

  // cursor of the tile being computed; start: largest b with cum[b] <= t0
  TileCursor cp;
  cp.t = t0;
  cp.b = 0;
  {
    int hi_b = B;                                              // cum[hi_b] > t0 always holds
    while (hi_b - cp.b > 1) {
      const int mid = (cp.b + hi_b) >> 1;
      if (uni(cum[mid]) <= t0) cp.b = mid; else hi_b = mid;
    }
  }
  enter_sequence(cp);
  {
    const uint32_t rem = t0 - uni(cum[cp.b]);
    cp.sib = rem / cp.tiles;
    cp.lt = rem - cp.sib * cp.tiles;
  }
  enter_strip(cp);
  cp.off = row_offset((int)cp.lt * 32, a.row_stride, a.block_stride, a.block_shift, a.block_mask);
  TileCursor ld = cp;                                          // cursor of the next tile to load
  // cursor of the strip whose Q operand is fetched next (first tile of a strip, or past the end)
  TileCursor qs = cp;
  auto next_strip = [&](TileCursor& cu) {                      // cu.t becomes >= t_end when done
    cu.t += cu.tiles - cu.lt;
    cu.lt = 0;
    if (cu.t < t_end) {
      if (++cu.sib == spb) {
        cu.sib = 0;
        ++cu.b;
        enter_sequence(cu);
      }
    }
  };

  // qop, lim: operand and row limit of the strip being computed; qnext, lnext: raw rows and limit
  // of the following strip, in flight for a whole strip before they are taken into use; qnext_nh:
  // how many of its columns are real; lnext_slot: its group's slot.  One of each per pass.
  u32x4 qop[P][4], qnext[P][4];
  Limit lnext[P];
  int lim[P], nh[P], qnext_nh[P];
  int g, pass0;                       // kv head and first pass of the strip being computed
  int qg = 0, qpass0 = 0, lnext_slot = 0;   // ... and of the strip whose rows are in flight
  // Q rows and limits of the P passes of a strip.  A pass without columns fetches those of pass 0,
  // which always has some (the wave's own first pass may be beyond the group's columns too, when
  // the waves of a worker carry more passes than the group has: its columns would belong to token
  // rows or heads that do not exist, past the end of q for the last sequence).
  auto fetch = [&](const TileCursor& cu, int b, int fg, int fpass0, const int (&fnh)[P]) {
#pragma unroll
    for (int i = 0; i < P; ++i) {
      const int pass = fnh[i] > 0 ? fpass0 + i : 0;
      load_q(qnext[i], a, b, fg, pass, fnh[i], hn, c);
      lnext[i] = load_limit(cu, b, fg, pass, fnh[i]);
    }
  };
  auto take = [&](const int (&tnh)[P], int slot) {
#pragma unroll
    for (int i = 0; i < P; ++i) {
      keep_real_heads(qop[i], qnext[i], tnh[i], hn);
      lim[i] = rows_of(lnext[i], slot);
    }
  };
  pass_of(cp.sib, g, pass0, nh);
  fetch(cp, cp.b, g, pass0, nh);
  take(nh, cp.slot);
  next_strip(qs);
#pragma unroll
  for (int i = 0; i < P; ++i) qnext_nh[i] = 0;
  // The Q rows of the following strip are fetched a whole strip ahead -- by a wave that carries one
  // pass.  With two passes the registers that would hold them are worth more than the stall: the
  // compiler parks what does not fit in the accumulator registers and moves it back and forth in
  // every tile; there the rows are fetched when the strip opens (one memory round trip per strip).
  constexpr bool kPrefetchQ = P == 1;
  if (kPrefetchQ && qs.t < t_end) {
    pass_of(qs.sib, qg, qpass0, qnext_nh);
    fetch(qs, qs.b, qg, qpass0, qnext_nh);
    lnext_slot = qs.slot;
  }

  f32x4 acc[P][8];
  float m[P], l[P];
#pragma unroll
  for (int i = 0; i < P; ++i) {
#pragma unroll
    for (int tcol = 0; tcol < 8; ++tcol) acc[i][tcol] = f32x4{0.f, 0.f, 0.f, 0.f};
    m[i] = kNegInf;
    l[i] = 0.f;
  }

  // One-launch step: the strips this wave wrote a record for (at most the one its share begins in
  // and the one it ends in), to be counted as arrived once the wave has nothing in flight.
  uint32_t part_strip[2] = {0u, 0u};                           // b * spb + sib
  int part_b[2] = {0, 0}, part_records[2] = {0, 0};
  int n_part = 0;

  // One tile of arithmetic; closes the record when the tile ends this wave's piece of the strip.
  // (the tile is in registers, or -- COOP -- in LDS)
  auto compute = [&](const TileRegs* regs, const TileLds* shared) {
    // (a pass without columns runs on a zero operand; its results are never stored)
    const bool strip_end = cp.lt + 1 == cp.tiles;
    if (cp.n > 0) {
      // (one-launch step: the strip's last tile is the new row, whose row number is n - 1)
      if constexpr (FUSED) {
        // the cached rows end at n - 2 (what a cache tile holds beyond is a clamped copy); the
        // strip's last tile is the new row alone, row number n - 1
        int upto[P];
#pragma unroll
        for (int i = 0; i < P; ++i) upto[i] = strip_end ? lim[i] : lim[i] - 1;
        process_tile<BF16, P>(*regs, qop, acc, m, l, a.scale_log2e,
                              strip_end ? cp.n - 1 : (int)cp.lt * 32, upto, c);
      } else if constexpr (COOP) {
        process_tile_lds<BF16, P>(*shared, qop, acc, m, l, a.scale_log2e, (int)cp.lt * 32, lim, hn, c);
      } else {
        process_tile<BF16, P>(*regs, qop, acc, m, l, a.scale_log2e, (int)cp.lt * 32, lim, c);
      }
    }
    if constexpr (FUSED) {
      // the append: the new row sits in this tile's registers (written by the first pass set only)
      if (strip_end && cp.n > 0 && cp.sib % (uint32_t)a.n_pass == 0 && wsub == 0) {
        const int64_t at = (int64_t)cp.slot * a.slot_stride + (int64_t)g * a.head_stride +
                           row_offset(cp.n - 1, a.row_stride, a.block_stride, a.block_shift, a.block_mask);
        store_new_row(*regs, reinterpret_cast<char*>(const_cast<uint16_t*>(a.k_cache) + at),
                      reinterpret_cast<char*>(const_cast<uint16_t*>(a.v_cache) + at), 0, lg);
      }
    }
    if (strip_end || cp.t + 1 == t_end) {
      const uint32_t strip_t0 = cp.t - cp.lt;                  // global index of the strip's tile 0
      int rec = (int)(gw - strip_t0 / share);
      if (cp.n > 0 || FUSED) {
        // the strip began inside this wave's share and ends here: nothing to merge
        // (one-launch step: a strip without rows is whole too, and its result is zero)
        const bool whole = a.out_kind != 0 && strip_end && strip_t0 >= t0;
#pragma unroll
        for (int i = 0; i < P; ++i) {
          if (nh[i] == 0) continue;
          if constexpr (COOP) {
            if (whole)
              store_final_natural<BF16>(a, cp.b, g, pass0 + i, nh[i], acc[i], l[i], hn, c);
            else
              store_record_natural(a, cp.b, g, pass0 + i, nh[i], rec, acc[i], m[i], l[i], hn, c);
          } else if (whole) {
            store_final<BF16>(a, cp.b, g, pass0 + i, nh[i], acc[i], l[i], hn, c);
          } else {
            store_record(a, cp.b, g, pass0 + i, nh[i], rec, acc[i], m[i], l[i], hn, c);
          }
        }
        if (FUSED && !whole) {
          // (slot 1 when slot 0 is taken: registers, not an indexed array)
          const uint32_t id = (uint32_t)cp.b * spb + cp.sib;
          const int records = (int)((strip_t0 + cp.tiles - 1) / share - strip_t0 / share) + 1;
          if (n_part == 0) {
            part_strip[0] = id;
            part_b[0] = cp.b;
            part_records[0] = records;
          } else {
            part_strip[1] = id;
            part_b[1] = cp.b;
            part_records[1] = records;
          }
          ++n_part;
        }
        rec = whole ? -1 : rec + 1;
      }
      if (!FUSED && strip_end && c == 0) {                     // records in use for these heads
#pragma unroll
        for (int i = 0; i < P; ++i)
          if (hn < nh[i]) a.ws_n[column_index(a, cp.b, g, pass0 + i, hn)] = rec;
      }
      if (cp.t + 1 < t_end) {                                  // the next tile opens a strip
#pragma unroll
        for (int i = 0; i < P; ++i) {
#pragma unroll
          for (int tcol = 0; tcol < 8; ++tcol) acc[i][tcol] = f32x4{0.f, 0.f, 0.f, 0.f};
          m[i] = kNegInf;
          l[i] = 0.f;
        }
        if constexpr (!kPrefetchQ) {
          pass_of(qs.sib, g, pass0, nh);                       // qs: the strip that opens
          fetch(qs, qs.b, g, pass0, nh);
          take(nh, qs.slot);
          next_strip(qs);
        } else {
        take(qnext_nh, lnext_slot);
        g = qg;
        pass0 = qpass0;
#pragma unroll
        for (int i = 0; i < P; ++i) nh[i] = qnext_nh[i];
        next_strip(qs);
        {
          // unconditional: when no strip follows, this strip's rows are fetched again (unused)
          const bool more = qs.t < t_end;
          const int qb = more ? qs.b : cp.b;
          pass_of(more ? qs.sib : cp.sib, qg, qpass0, qnext_nh);
          if constexpr (GROUPED) {
            fetch(qs, qb, qg, qpass0, qnext_nh);
          } else {
#pragma unroll
            for (int i = 0; i < P; ++i) {
              // (a pass without columns fetches pass 0's rows, as fetch() does)
              load_q(qnext[i], a, qb, qg, qnext_nh[i] > 0 ? qpass0 + i : 0, qnext_nh[i], hn, c);
              lnext[i] = Limit{0, more ? qs.n : cp.n};
            }
          }
          lnext_slot = more ? qs.slot : cp.slot;
        }
        }
      }
    }
  };

  if constexpr (COOP) {
    // Each wave keeps its shares of the next two tiles in flight (four were measured: no faster, and
    // two leave the registers for two waves per SIMD).  Per tile: put the share that has arrived
    // into the LDS tile, ask for the share two tiles on, meet the other waves,
    // compute from LDS.  Two LDS tiles and one barrier per tile: the tile written before
    // barrier i is read after it, and is written again only after barrier i + 1, which no wave
    // passes before all have finished reading.  The waves run the same tiles to the same end,
    // so every wave reaches every barrier.
    __shared__ TileLds exchange[2];
    auto next_part = [&](PartRegs<kPartWaves>& pr) {
      if (ld.t + 1 < t_end) advance(ld);
      issue_part(pr, ld);
    };
    PartRegs<kPartWaves> p0, p1;
    issue_part(p0, ld);
    next_part(p1);
    int buf = 0;
    // (Steps come two to a loop iteration, one per register share, and the loop has a single
    // exit: a step past the worker's last tile still puts, loads -- the last position again -- and
    // meets the others, and skips the arithmetic.  With an exit after every step the paths that
    // leave would join the loop's back edge, and the wait before the first put of an iteration
    // would be for everything in flight instead of for that share.)
    bool live = true;
    auto step = [&](PartRegs<kPartWaves>& pr) {
      put_part<kPartWaves>(exchange[buf], pr, (int)wave, lg);
      next_part(pr);
      __syncthreads();
      if (live) {
        compute(nullptr, &exchange[buf]);
        if (cp.t + 1 >= t_end) live = false; else advance(cp);
      }
      buf ^= 1;
    };
    do {
      step(p0);
      step(p1);
    } while (live);
  } else {
    // Two register tiles: one is in flight while the other is computed.  Loads are issued
    // unconditionally (past the end of the share the last position is loaded again, from cache) so
    // that every wait count is exact.
    auto load_next = [&](TileRegs& regs) {
      if (ld.t + 1 < t_end) advance(ld);
      issue(regs, ld);
    };
    TileRegs ta, tb;
    issue(ta, ld);
    while (true) {
      load_next(tb);
      compute(&ta, nullptr);
      if (cp.t + 1 >= t_end) break;
      advance(cp);
      load_next(ta);
      compute(&tb, nullptr);
      if (cp.t + 1 >= t_end) break;
      advance(cp);
    }
  }

  if constexpr (FUSED) {
    // The merge, in the same launch: a strip that several waves covered is finished by the wave
    // whose record arrives last.  The wave has no tile in flight any more, so waiting for its own
    // stores costs nothing here; its records are in memory before the arrival is counted, the
    // counter says how many records were there before, and the wave that finds all the others
    // there merges (reading them at device scope).
    // Nobody waits for anybody.  The last arrival also clears the counter for the next launch.
    if (n_part > 0) {
      // (records are written through to memory, so "visible" only means "the stores have
      // completed": a workgroup-scope release waits for them without flushing the L2)
      __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        if (k < n_part) {
          int before = 0;
          // (waves that share a strip's rows carry different passes: a counter each)
          if (lane == 0) before = atomicAdd(a.arrive + part_strip[k] * n_share + wave % n_share, 1);
          before = __builtin_amdgcn_readfirstlane(before);
          if (before + 1 == part_records[k]) {
            if (lane == 0)
              __hip_atomic_store(a.arrive + part_strip[k] * n_share + wave % n_share, 0,
                                 __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
            int mg, mpass0, mnh[P];
            pass_of(part_strip[k] % spb, mg, mpass0, mnh);
#pragma unroll
            for (int i = 0; i < P; ++i)
              if (mnh[i] > 8)
                merge_columns<BF16, 8, 3>(a, part_b[k], mg, mpass0 + i, mnh[i], part_records[k], lane);
              else if (mnh[i] > 0)
                merge_columns<BF16, 4, 6>(a, part_b[k], mg, mpass0 + i, mnh[i], part_records[k], lane);
          }
        }
      }
    }
  }
}

// The one-launch step for SMALL batches: one workgroup per strip (sequence, kv head, head pass).
//
// When a batch has fewer strips than the chip has wave slots, cutting the strips into equal shares
// (above) leaves every strip in pieces on different compute units, and putting the pieces together
// costs memory round trips that are as long as the streaming itself.  Here the WAVES waves of one
// workgroup take a strip's tiles in turn (wave w: tiles w, w + WAVES, ...), keep their own running
// sums, and merge them through LDS: no workspace, no counters, no second kernel.  The appended row
// is the strip's last tile, loaded from k_new / v_new and written to the caches from registers, as
// in the balanced one-launch kernel.  ctx_len[] holds the positions of the new rows.
//
// LDS: WAVES x 16 head columns x (128 + 4) floats of scaled partial rows, and the (exponent, sum)
// pairs: 68 KB for eight waves.
template <bool BF16, int WAVES>
__global__ __launch_bounds__(WAVES * 64, 2) void attn_mfma_strip_kernel(const AttnArgs a) {
  constexpr int kPitch = kHeadDim + 4;                         // floats per head column in LDS
  __shared__ float rows_lds[WAVES][16][kPitch];
  __shared__ float m_lds[WAVES][16], l_lds[WAVES][16];
  auto uni = [](int x) { return __builtin_amdgcn_readfirstlane(x); };
  const int tid = threadIdx.x, lane = tid & 63, wave = uni(tid >> 6);
  const int hn = lane & 15, c = lane >> 4;

  // strip of this workgroup: pass fastest, then kv head, then sequence
  int rest = (int)blockIdx.x;
  const int pass = rest % a.n_pass;
  rest /= a.n_pass;
  const int g = rest % a.n_kv_heads, b = rest / a.n_kv_heads;
  const int left = a.group - pass * a.heads_per_pass;
  const int nh = left < a.heads_per_pass ? left : a.heads_per_pass;

  const int slot = uni(a.slot_id[b]), pos = uni(a.ctx_len[b]);
  const bool bad_slot = slot < 0 || slot >= a.n_slots, bad_pos = pos < 0 || pos >= a.row_limit;
  if ((bad_slot || bad_pos) && a.dev_status && g == 0 && pass == 0 && tid == 0)
    atomicOr(a.dev_status, (bad_slot ? 1 : 0) | (bad_pos ? 2 : 0));
  const int n = bad_slot || bad_pos ? 0 : pos + 1;             // rows attended; row n - 1 is the new one
  const int tiles = n > 0 ? ((n - 1 + 31) >> 5) + 1 : 0;       // cached rows in tiles, then the new row

  u32x4 qop[1][4];
  {
    u32x4 qraw[4];
    load_q(qraw, a, b, g, pass, nh, hn, c);
    keep_real_heads(qop[0], qraw, nh, hn);
  }
  f32x4 acc[1][8];
#pragma unroll
  for (int tcol = 0; tcol < 8; ++tcol) acc[0][tcol] = f32x4{0.f, 0.f, 0.f, 0.f};
  float m[1] = {kNegInf}, l[1] = {0.f};

  const LaneGeom lg = lane_geom(hn, c);
  const uint32_t row_bytes = (uint32_t)a.row_stride * 2u;
  const int64_t strip = (int64_t)(n > 0 ? slot : 0) * a.slot_stride + (int64_t)g * a.head_stride;
  const int64_t from = (int64_t)b * a.new_batch_stride + (int64_t)g * kHeadDim;
  // tile t of the strip; past this wave's last one the same tile is loaded again (from cache), so
  // that every wait count is exact
  auto issue = [&](TileRegs& regs, int t) {
    if (t + 1 == tiles) {
      load_tile<true>(regs, reinterpret_cast<const char*>(a.k_new + from),
                      reinterpret_cast<const char*>(a.v_new + from), row_bytes, 1, lg);
    } else {
      const int64_t at = strip + row_offset(t * 32, a.row_stride, a.block_stride, a.block_shift, a.block_mask);
      load_tile<true>(regs, reinterpret_cast<const char*>(a.k_cache + at),
                      reinterpret_cast<const char*>(a.v_cache + at), row_bytes, n - 1 - t * 32, lg);
    }
  };
  auto compute = [&](const TileRegs& regs, int t) {
    const bool last = t + 1 == tiles;
    const int upto[1] = {last ? n : n - 1};
    process_tile<BF16, 1>(regs, qop, acc, m, l, a.scale_log2e, last ? n - 1 : t * 32, upto, c);
    if (last && pass == 0) {                                   // the append, from the tile's registers
      const int64_t at = strip + row_offset(n - 1, a.row_stride, a.block_stride, a.block_shift, a.block_mask);
      store_new_row(regs, reinterpret_cast<char*>(const_cast<uint16_t*>(a.k_cache) + at),
                    reinterpret_cast<char*>(const_cast<uint16_t*>(a.v_cache) + at), 0, lg);
    }
  };
  if (wave < tiles) {
    // this wave's tiles: wave, wave + WAVES, ...; two register tiles, one in flight
    const int last_mine = wave + (tiles - 1 - wave) / WAVES * WAVES;
    TileRegs ta, tb;
    issue(ta, wave);
    for (int t = wave;; t += 2 * WAVES) {
      issue(tb, t + WAVES <= last_mine ? t + WAVES : last_mine);
      compute(ta, t);
      if (t + WAVES > last_mine) break;
      issue(ta, t + 2 * WAVES <= last_mine ? t + 2 * WAVES : last_mine);
      compute(tb, t + WAVES);
      if (t + 2 * WAVES > last_mine) break;
    }
  }

  // merge through LDS: common exponent per head column, every wave's rows scaled to it
  l[0] = rows_sum(l[0]);
  if (c == 0) {
    m_lds[wave][hn] = m[0];
    l_lds[wave][hn] = l[0];
  }
  __syncthreads();
  float top = kNegInf;
#pragma unroll
  for (int w = 0; w < WAVES; ++w) top = fmaxf(top, l_lds[w][hn] > 0.f ? m_lds[w][hn] : kNegInf);
  const float mine = l[0] > 0.f && top != kNegInf ? fast_exp2(m[0] - top) : 0.f;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    // register i of column tile t is column 32c + 8i + t: eight consecutive columns per i
    f32x4 lo = {acc[0][0][i], acc[0][1][i], acc[0][2][i], acc[0][3][i]};
    f32x4 hi = {acc[0][4][i], acc[0][5][i], acc[0][6][i], acc[0][7][i]};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      lo[e] = mine > 0.f ? lo[e] * mine : 0.f;                 // (a wave without rows holds zeros)
      hi[e] = mine > 0.f ? hi[e] * mine : 0.f;
    }
    *reinterpret_cast<f32x4*>(&rows_lds[wave][hn][32 * c + 8 * i]) = lo;
    *reinterpret_cast<f32x4*>(&rows_lds[wave][hn][32 * c + 8 * i + 4]) = hi;
  }
  __syncthreads();
  // thread -> (head column, four output columns); WAVES * 64 threads cover 16 x 32 such pieces
  typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
  for (int piece = tid; piece < 16 * 32; piece += WAVES * 64) {
    const int head = piece >> 5, col = (piece & 31) * 4;
    if (head >= nh) continue;
    float peak = kNegInf;
#pragma unroll
    for (int w = 0; w < WAVES; ++w) peak = fmaxf(peak, l_lds[w][head] > 0.f ? m_lds[w][head] : kNegInf);
    float total = 0.f;
    f32x4 x = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int w = 0; w < WAVES; ++w) {
      const float lw = l_lds[w][head];
      if (lw > 0.f) {
        total = fmaf(fast_exp2(m_lds[w][head] - peak), lw, total);
        x += *reinterpret_cast<const f32x4*>(&rows_lds[w][head][col]);
      }
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) x[e] = total > 0.f ? x[e] / total : 0.f;
    const int64_t row = column_index(a, b, g, pass, head);
    if (a.out_kind == 1) {
      *reinterpret_cast<f32x4*>(static_cast<float*>(a.out) + row * kHeadDim + col) = x;
    } else {
      const u32x2 w2 = {pack2<BF16>(x[0], x[1]), pack2<BF16>(x[2], x[3])};
      *reinterpret_cast<u32x2*>(static_cast<uint16_t*>(a.out) + row * kHeadDim + col) = w2;
    }
  }
}

}  // namespace gh

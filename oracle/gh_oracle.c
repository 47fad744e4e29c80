/*
 * gh_oracle.c -- plain CPU float64 reference for the Tier-2 attention step.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing in the product path may call, link or
 * import this file; it exists so that the GPU kernels can be checked against
 * an implementation that is slow and obviously correct.  It shares no source,
 * header, table or helper with the HIP library.
 *
 * What it computes (paper Section 2.1, stage F2(C_k, qkv) -> C_k, x'_k;
 * Appendix A, Table 5 rows "Q_i^T.K_i" and "A_i^T.V_i"; Section 4.3:
 * standard multi-head attention with grouped-query support, Table 1 symbols
 * H, H_kv, D/H):
 *
 *   append : the step's new key row and value row of every KV head are
 *            copied into the sequence's context slot at the position of the
 *            latest token (Section 4.1.3: the batch state object carries the
 *            context location identifier and that position).
 *   attend : for sequence b and query head h, with g = h / (H / H_kv),
 *              s_r  = scale * sum_j q[b,h,j] * K[slot_b, g, r, j]   r < n_b
 *              w_r  = exp(s_r - max_r s_r) / sum_r exp(s_r - max_r s_r)
 *              out[b,h,:] = sum_r w_r * V[slot_b, g, r, :]
 *            all arithmetic in double; each 16-bit input is widened exactly.
 *
 * The split form (footnote of Section 2.2: attention parallelised along the
 * sequence) is exposed separately as gho_partial / gho_merge so that the
 * merge rule can be pinned against the unsplit definition:
 *   partial over rows [r0,r1): t_r = s_r*log2(e), m = max t_r,
 *                              l = sum 2^(t_r-m), o = sum 2^(t_r-m) V_r
 *   merge: M = max_c m_c, out = sum_c 2^(m_c-M) o_c / sum_c 2^(m_c-M) l_c,
 *          chunks with no rows contribute nothing.
 *
 * Parity pins (tests/test_oracle_pins.py): identical keys -> mean of V,
 * length 1 -> that V row, joint row permutation, brute-force enumeration in
 * pure Python, constant V, linearity in V, key-shift invariance, one-hot
 * limit, GQA == MHA with replicated KV heads, split/merge identity, a float64
 * library softmax-attention on small shapes, batch/head independence, and a
 * byte-for-byte append check.  No function here is "parity unpinned".
 *
 * Threads: OpenMP over (sequence, head) only; each output vector is produced
 * by one thread in a fixed order, so the thread count cannot change a bit.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { GHO_F16 = 0, GHO_BF16 = 1 };

typedef struct {
  int32_t batch;         /* B                                    */
  int32_t n_q_heads;     /* H                                    */
  int32_t n_kv_heads;    /* H_kv, divides H                      */
  int32_t head_dim;      /* d = D/H (any positive value here)    */
  int32_t dtype;         /* GHO_F16 or GHO_BF16                  */
  int32_t n_slots;       /* slots in the cache                   */
  int32_t slot_capacity; /* rows per slot                        */
  int64_t slot_stride;   /* cache strides, in 16-bit elements    */
  int64_t head_stride;
  int64_t row_stride;
  double scale;          /* softmax scaling of the scores        */
  int32_t block_rows;    /* 0, or rows per block of a blocked layout */
  int64_t block_stride;  /* elements between blocks of one head      */
} gho_problem;

/* Offset of row r inside a (slot, head) strip.  Plain layouts: r * row_stride.  Blocked layouts
 * (pages that hold block_rows consecutive rows of every head, each head's rows together):
 * block r / block_rows starts at that multiple of block_stride, rows inside it are row_stride
 * apart.  A storage choice only; no arithmetic depends on it. */
static int64_t row_offset(const gho_problem* p, int64_t r) {
  if (p->block_rows <= 0) return r * p->row_stride;
  return (r / p->block_rows) * p->block_stride + (r % p->block_rows) * p->row_stride;
}

/* IEEE 754 binary16 -> double, exact (subnormals, inf, NaN included). */
double gho_f16_to_f64(uint16_t h) {
  int sign = (h >> 15) & 1;
  int ex = (h >> 10) & 0x1f;
  int man = h & 0x3ff;
  double v;
  if (ex == 0) {
    v = ldexp((double)man, -24);            /* subnormal: man * 2^-10 * 2^-14 */
  } else if (ex == 31) {
    v = man ? NAN : INFINITY;
  } else {
    v = ldexp((double)(man | 0x400), ex - 25); /* (1+man/1024) * 2^(ex-15) */
  }
  return sign ? -v : v;
}

/* bfloat16 (upper half of binary32) -> double, exact. */
double gho_bf16_to_f64(uint16_t h) {
  int sign = (h >> 15) & 1;
  int ex = (h >> 7) & 0xff;
  int man = h & 0x7f;
  double v;
  if (ex == 0) {
    v = ldexp((double)man, -133);           /* man * 2^-7 * 2^-126 */
  } else if (ex == 255) {
    v = man ? NAN : INFINITY;
  } else {
    v = ldexp((double)(man | 0x80), ex - 134); /* (1+man/128) * 2^(ex-127) */
  }
  return sign ? -v : v;
}

static double widen(int dtype, uint16_t x) {
  return dtype == GHO_BF16 ? gho_bf16_to_f64(x) : gho_f16_to_f64(x);
}

int gho_num_threads(void) {
#ifdef _OPENMP
  return omp_get_max_threads();
#else
  return 1;
#endif
}

void gho_set_num_threads(int n) {
#ifdef _OPENMP
  if (n > 0) omp_set_num_threads(n);
#else
  (void)n;
#endif
}

/*
 * Append (stage F2's update of C_k).  Host mirror of the cache; k_new, v_new
 * are [B, H_kv, d] contiguous.  Sequences whose slot id or position fall
 * outside the cache are skipped and reported through *n_skipped.
 */
void gho_kv_append(const gho_problem* p, uint16_t* k_cache, uint16_t* v_cache,
                   const uint16_t* k_new, const uint16_t* v_new,
                   const int32_t* slot_id, const int32_t* pos,
                   int32_t* n_skipped) {
  int32_t skipped = 0;
  const int64_t d = p->head_dim;
  for (int32_t b = 0; b < p->batch; ++b) {
    if (slot_id[b] < 0 || slot_id[b] >= p->n_slots || pos[b] < 0 ||
        pos[b] >= p->slot_capacity) {
      ++skipped;
      continue;
    }
    for (int32_t g = 0; g < p->n_kv_heads; ++g) {
      int64_t dst = (int64_t)slot_id[b] * p->slot_stride +
                    (int64_t)g * p->head_stride + row_offset(p, pos[b]);
      int64_t src = ((int64_t)b * p->n_kv_heads + g) * d;
      memcpy(k_cache + dst, k_new + src, (size_t)d * sizeof(uint16_t));
      memcpy(v_cache + dst, v_new + src, (size_t)d * sizeof(uint16_t));
    }
  }
  if (n_skipped) *n_skipped = skipped;
}

/* Scores s_r, r0 <= r < r1, of (sequence b, head h) into s[0 .. r1-r0). */
static void scores(const gho_problem* p, const uint16_t* q,
                   const uint16_t* k_cache, int32_t slot, int32_t b, int32_t h,
                   int32_t r0, int32_t r1, double* s) {
  const int32_t G = p->n_q_heads / p->n_kv_heads;
  const int32_t g = h / G;
  const int64_t d = p->head_dim;
  const uint16_t* qv = q + ((int64_t)b * p->n_q_heads + h) * d;
  for (int32_t r = r0; r < r1; ++r) {
    const uint16_t* kr = k_cache + (int64_t)slot * p->slot_stride +
                         (int64_t)g * p->head_stride + row_offset(p, r);
    double acc = 0.0;
    for (int64_t j = 0; j < d; ++j)
      acc += widen(p->dtype, qv[j]) * widen(p->dtype, kr[j]);
    s[r - r0] = p->scale * acc;
  }
}

/*
 * Attention by its definition.  q is [B, H, d]; ctx_len[b] = n_b rows
 * attended (after the append); out is [B, H, d] double.  n_b == 0 or a slot id
 * outside [0, n_slots) gives zeros.
 */
void gho_decode_attention(const gho_problem* p, const uint16_t* q,
                          const uint16_t* k_cache, const uint16_t* v_cache,
                          const int32_t* slot_id, const int32_t* ctx_len,
                          double* out) {
  const int32_t H = p->n_q_heads;
  const int32_t G = H / p->n_kv_heads;
  const int64_t d = p->head_dim;
  const int64_t items = (int64_t)p->batch * H;
#pragma omp parallel for schedule(dynamic, 1)
  for (int64_t it = 0; it < items; ++it) {
    const int32_t b = (int32_t)(it / H), h = (int32_t)(it % H);
    const int32_t n = ctx_len[b], slot = slot_id[b], g = h / G;
    double* o = out + it * d;
    for (int64_t j = 0; j < d; ++j) o[j] = 0.0;
    if (n <= 0) continue;
    /* a context location that does not exist holds no rows: the sequence is skipped, as the
       append skips it (Section 4.1.3 addresses a sequence by its context location) */
    if (slot < 0 || slot >= p->n_slots) continue;
    double* s = (double*)malloc((size_t)n * sizeof(double));
    scores(p, q, k_cache, slot, b, h, 0, n, s);
    double mx = s[0];
    for (int32_t r = 1; r < n; ++r) mx = s[r] > mx ? s[r] : mx;
    double Z = 0.0;
    for (int32_t r = 0; r < n; ++r) {
      s[r] = exp(s[r] - mx);
      Z += s[r];
    }
    for (int32_t r = 0; r < n; ++r) {
      const double w = s[r] / Z;
      const uint16_t* vr = v_cache + (int64_t)slot * p->slot_stride +
                           (int64_t)g * p->head_stride + row_offset(p, r);
      for (int64_t j = 0; j < d; ++j) o[j] += w * widen(p->dtype, vr[j]);
    }
    free(s);
  }
}

/*
 * Partial softmax result of (sequence b, head h) over rows [r0, r1), in the
 * base-2 form that the merge rule uses.  Empty range: m = -inf, l = 0, o = 0.
 */
void gho_partial(const gho_problem* p, const uint16_t* q,
                 const uint16_t* k_cache, const uint16_t* v_cache,
                 const int32_t* slot_id, int32_t b, int32_t h, int32_t r0,
                 int32_t r1, double* m_out, double* l_out, double* o) {
  const int32_t G = p->n_q_heads / p->n_kv_heads;
  const int32_t g = h / G, slot = slot_id[b];
  const int64_t d = p->head_dim;
  for (int64_t j = 0; j < d; ++j) o[j] = 0.0;
  if (r1 <= r0 || slot < 0 || slot >= p->n_slots) {
    *m_out = -INFINITY;
    *l_out = 0.0;
    return;
  }
  const int32_t n = r1 - r0;
  double* t = (double*)malloc((size_t)n * sizeof(double));
  scores(p, q, k_cache, slot, b, h, r0, r1, t);
  const double log2e = 1.4426950408889634074;
  for (int32_t r = 0; r < n; ++r) t[r] *= log2e;
  double m = t[0];
  for (int32_t r = 1; r < n; ++r) m = t[r] > m ? t[r] : m;
  double l = 0.0;
  for (int32_t r = 0; r < n; ++r) {
    const double w = exp2(t[r] - m);
    l += w;
    const uint16_t* vr = v_cache + (int64_t)slot * p->slot_stride +
                         (int64_t)g * p->head_stride +
                         row_offset(p, r0 + r);
    for (int64_t j = 0; j < d; ++j) o[j] += w * widen(p->dtype, vr[j]);
  }
  free(t);
  *m_out = m;
  *l_out = l;
}

/*
 * Merge of n_chunks partial results of one (sequence, head):
 * m[c], l[c], o[c*d .. c*d+d).  All chunks empty -> zeros.
 */
void gho_merge(int32_t n_chunks, int32_t d, const double* m, const double* l,
               const double* o, double* out) {
  double M = -INFINITY;
  for (int32_t c = 0; c < n_chunks; ++c)
    if (l[c] > 0.0 && m[c] > M) M = m[c];
  for (int32_t j = 0; j < d; ++j) out[j] = 0.0;
  if (M == -INFINITY) return;
  double L = 0.0;
  for (int32_t c = 0; c < n_chunks; ++c) {
    if (!(l[c] > 0.0)) continue;
    const double w = exp2(m[c] - M);
    L += w * l[c];
    for (int32_t j = 0; j < d; ++j) out[j] += w * o[(int64_t)c * d + j];
  }
  for (int32_t j = 0; j < d; ++j) out[j] /= L;
}

/*
 * Runs the CPU oracle on a problem read from a file and writes what it computed, so that a build
 * of oracle/gh_oracle.c under AddressSanitizer / UndefinedBehaviorSanitizer can be compared bit
 * for bit with the ordinary build (tests/test_sanitized_host_code.py).  Every array is read into
 * a heap block of exactly its size, so a read or write one element outside is caught.
 *
 * Input (little endian): int64 header[16] = B, H, H_kv, d, dtype, n_slots, capacity, slot_stride,
 * head_stride, row_stride, block_rows, block_stride, cache_elems, split_row, 0, 0; double scale;
 * uint16 q[B*H*d], k_new[B*H_kv*d], v_new[B*H_kv*d], k_cache[cache_elems], v_cache[cache_elems];
 * int32 slot_id[B], pos[B], ctx_len[B].
 * Output: int32 skipped; double out[B*H*d]; double merged[B*H*d] (each head's rows cut at
 * split_row, the two partial results merged); uint16 k_cache, v_cache after the append.
 */
#include <stdio.h>

#include "../../oracle/gh_oracle.c"

static void* read_block(FILE* f, size_t bytes) {
  void* p = malloc(bytes ? bytes : 1);
  if (!p || fread(p, 1, bytes, f) != bytes) {
    fprintf(stderr, "oracle_driver: short read\n");
    exit(2);
  }
  return p;
}

int main(int argc, char** argv) {
  if (argc != 3) return 2;
  FILE* f = fopen(argv[1], "rb");
  if (!f) return 2;
  int64_t h[16];
  double scale;
  if (fread(h, sizeof h, 1, f) != 1 || fread(&scale, sizeof scale, 1, f) != 1) return 2;
  gho_problem p;
  memset(&p, 0, sizeof p);
  p.batch = (int32_t)h[0];
  p.n_q_heads = (int32_t)h[1];
  p.n_kv_heads = (int32_t)h[2];
  p.head_dim = (int32_t)h[3];
  p.dtype = (int32_t)h[4];
  p.n_slots = (int32_t)h[5];
  p.slot_capacity = (int32_t)h[6];
  p.slot_stride = h[7];
  p.head_stride = h[8];
  p.row_stride = h[9];
  p.scale = scale;
  p.block_rows = (int32_t)h[10];
  p.block_stride = h[11];
  const size_t B = (size_t)h[0], H = (size_t)h[1], Hkv = (size_t)h[2], d = (size_t)h[3];
  const size_t cache = (size_t)h[12];
  const int32_t split_row = (int32_t)h[13];
  uint16_t* q = read_block(f, B * H * d * 2);
  uint16_t* k_new = read_block(f, B * Hkv * d * 2);
  uint16_t* v_new = read_block(f, B * Hkv * d * 2);
  uint16_t* k_cache = read_block(f, cache * 2);
  uint16_t* v_cache = read_block(f, cache * 2);
  int32_t* slot_id = read_block(f, B * 4);
  int32_t* pos = read_block(f, B * 4);
  int32_t* ctx_len = read_block(f, B * 4);
  fclose(f);

  int32_t skipped = -1;
  gho_kv_append(&p, k_cache, v_cache, k_new, v_new, slot_id, pos, &skipped);
  double* out = malloc(B * H * d * sizeof(double) + 8);
  gho_decode_attention(&p, q, k_cache, v_cache, slot_id, ctx_len, out);

  double* merged = malloc(B * H * d * sizeof(double) + 8);
  double* po = malloc(2 * d * sizeof(double));
  for (size_t b = 0; b < B; ++b) {
    for (size_t hh = 0; hh < H; ++hh) {
      double m[2], l[2];
      int32_t n = ctx_len[b];
      if (slot_id[b] < 0 || slot_id[b] >= p.n_slots || n < 0) n = 0;
      const int32_t cut = split_row < n ? split_row : n;
      gho_partial(&p, q, k_cache, v_cache, slot_id, (int32_t)b, (int32_t)hh, 0, cut, &m[0], &l[0], po);
      gho_partial(&p, q, k_cache, v_cache, slot_id, (int32_t)b, (int32_t)hh, cut, n, &m[1], &l[1], po + d);
      gho_merge(2, (int32_t)d, m, l, po, merged + (b * H + hh) * d);
    }
  }

  f = fopen(argv[2], "wb");
  if (!f) return 2;
  fwrite(&skipped, 4, 1, f);
  fwrite(out, sizeof(double), B * H * d, f);
  fwrite(merged, sizeof(double), B * H * d, f);
  fwrite(k_cache, 2, cache, f);
  fwrite(v_cache, 2, cache, f);
  fclose(f);
  free(q); free(k_new); free(v_new); free(k_cache); free(v_cache);
  free(slot_id); free(pos); free(ctx_len); free(out); free(merged); free(po);

  /* the two decoders over every bit pattern: checksum of the finite values, count of the others */
  double sum[2] = {0.0, 0.0};
  int odd[2] = {0, 0};
  for (uint32_t u = 0; u < 65536; ++u) {
    const double a = gho_f16_to_f64((uint16_t)u), c = gho_bf16_to_f64((uint16_t)u);
    if (isfinite(a)) sum[0] += fabs(a); else ++odd[0];
    if (isfinite(c)) sum[1] += fabs(c) * 1e-30; else ++odd[1];
  }
  printf("decoders %a %d %a %d\n", sum[0], odd[0], sum[1], odd[1]);
  return 0;
}

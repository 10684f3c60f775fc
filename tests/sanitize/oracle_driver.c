/* Drives every entry point of the CPU oracle on small inputs with exact-size heap buffers.  Built by
 * tests/test_sanitizers.py with gcc -fsanitize=address,undefined: an out-of-bounds access, a use of freed memory, a
 * signed overflow, a bad shift or a misaligned access inside the oracle aborts the run.  Prints "ok <checksum>". */
#include <math.h>
#include <stdint.h>
#include <stdio.h>
#include <stdlib.h>
#include <string.h>

#include "akvq_oracle.h"

static uint64_t state = 0x9E3779B97F4A7C15ull;
static uint32_t next_u32(void) {
  state ^= state << 13; state ^= state >> 7; state ^= state << 17;
  return (uint32_t)(state >> 32);
}
static uint16_t rand_half(float scale) { /* roughly uniform in [-scale, scale] */
  float f = ((float)(next_u32() & 0xFFFF) / 32768.0f - 1.0f) * scale;
  return orc_float_to_half_rne(f);
}
static void *xalloc(size_t n) { void *p = malloc(n ? n : 1); if (!p) abort(); memset(p, 0, n); return p; }

typedef struct { orc_cache c; uint32_t *fine; uint16_t *k_win, *v_win; int W; } cache_t;

static cache_t make_cache(int B, int Hkv, int G, int T_cap, int S_cap, int W, int tiered) {
  cache_t x; memset(&x, 0, sizeof(x));
  size_t bh = (size_t)B * Hkv;
  x.c.B = B; x.c.Hkv = Hkv; x.c.G = G; x.c.T_cap = T_cap; x.c.S_cap = S_cap; x.c.T_len = 0;
  x.c.k_codes = xalloc(bh * (T_cap / 32) * 256 * 4); x.c.v_codes = xalloc(bh * (T_cap / 32) * 256 * 4);
  x.c.k_meta = xalloc(bh * T_cap * (128 / G) * 4);   x.c.v_meta = xalloc(bh * T_cap * (128 / G) * 4);
  x.c.k_sal = xalloc(bh * S_cap * 128 * 2);          x.c.v_sal = xalloc(bh * S_cap * 128 * 2);
  x.c.sal_idx = xalloc(bh * S_cap * 4);              x.c.sal_cnt = xalloc(bh * 4);
  if (tiered) x.fine = xalloc((size_t)B * (T_cap / 32) * 4);
  x.W = W;
  if (W) { x.k_win = xalloc(bh * W * 128 * 2); x.v_win = xalloc(bh * W * 128 * 2); }
  return x;
}
static void free_cache(cache_t *x) {
  free(x->c.k_codes); free(x->c.v_codes); free(x->c.k_meta); free(x->c.v_meta); free(x->c.k_sal); free(x->c.v_sal);
  free(x->c.sal_idx); free(x->c.sal_cnt); free(x->fine); free(x->k_win); free(x->v_win);
}

static double run_case(int B, int Hq, int Hkv, int G, int T, int W_score, int top_k, int window, int tiered) {
  const int T_cap = (2 * T + 64 + 63) / 64 * 64, S_cap = 64;
  size_t n_kv = (size_t)B * Hkv * T * 128;
  uint16_t *k = xalloc(n_kv * 2), *v = xalloc(n_kv * 2), *qt = xalloc((size_t)B * Hq * W_score * 128 * 2);
  uint16_t *q = xalloc((size_t)B * Hq * 128 * 2);
  uint8_t *is_text = xalloc((size_t)B * T);
  for (size_t i = 0; i < n_kv; ++i) { k[i] = rand_half(i % 128 == 5 ? 40.0f : 2.0f); v[i] = rand_half(2.0f); }
  for (size_t i = 0; i < (size_t)B * Hq * W_score * 128; ++i) qt[i] = rand_half(2.0f);
  for (size_t i = 0; i < (size_t)B * Hq * 128; ++i) q[i] = rand_half(2.0f);
  for (int b = 0; b < B; ++b) for (int t = 0; t < T; ++t) is_text[(size_t)b * T + t] = (t < 3 || t >= T - 2 || t % 11 == 0);
  double sum = 0.0;
  double *out = xalloc((size_t)B * Hq * 128 * 8), *lse = xalloc((size_t)B * Hq * 8);
  double *mass = xalloc((size_t)B * Hkv * T * 8);

  /* text-salient cache, plain append in two pieces, decode */
  cache_t a = make_cache(B, Hkv, G, T_cap, S_cap, 0, 0);
  orc_select_tsa(&a.c, is_text, T);
  int first = T / 3 + 1;
  uint16_t *k1 = xalloc((size_t)B * Hkv * first * 128 * 2), *v1 = xalloc((size_t)B * Hkv * first * 128 * 2);
  uint16_t *k2 = xalloc((size_t)B * Hkv * (T - first) * 128 * 2), *v2 = xalloc((size_t)B * Hkv * (T - first) * 128 * 2);
  for (int bh = 0; bh < B * Hkv; ++bh) {
    memcpy(k1 + (size_t)bh * first * 128, k + (size_t)bh * T * 128, (size_t)first * 256);
    memcpy(v1 + (size_t)bh * first * 128, v + (size_t)bh * T * 128, (size_t)first * 256);
    memcpy(k2 + (size_t)bh * (T - first) * 128, k + ((size_t)bh * T + first) * 128, (size_t)(T - first) * 256);
    memcpy(v2 + (size_t)bh * (T - first) * 128, v + ((size_t)bh * T + first) * 128, (size_t)(T - first) * 256);
  }
  orc_quantize_append(&a.c, k1, v1, first, 0.8f, ORC_ROT_K | ORC_ROT_V); a.c.T_len = first;
  orc_quantize_append(&a.c, k2, v2, T - first, 0.8f, ORC_ROT_K | ORC_ROT_V); a.c.T_len = T;
  orc_decode_attention(&a.c, Hq, q, 0.0884, ORC_ROT_Q | ORC_ROT_OUT, out, lse);
  for (int i = 0; i < B * Hq * 128; ++i) sum += out[i];
  orc_decode_attention_one(&a.c, Hq, B - 1, Hq - 1, q + ((size_t)(B - 1) * Hq + Hq - 1) * 128, 0.0884, 0, out, lse);
  sum += out[0] + orc_get_code(&a.c, 1, B - 1, Hkv - 1, T - 1, 127);

  /* pivot-salient (per head and token-level), un-rotated variants */
  cache_t p = make_cache(B, Hkv, G, T_cap, S_cap, 0, 0);
  orc_select_psa(&p.c, Hq, qt, k, T, W_score, top_k, 0.0884, mass);
  orc_select_psa_shared(&p.c, Hq, qt, k, T, W_score, top_k, 0.0884, NULL);
  orc_quantize_append(&p.c, k, v, T, 1.0f, 0); p.c.T_len = T;
  orc_decode_attention(&p.c, Hq, q, 0.0884, 0, out, NULL);
  for (int i = 0; i < B * Hq * 128; ++i) sum += out[i];
  for (size_t i = 0; i < (size_t)B * Hkv * T; ++i) sum += mass[i];

  /* tiers + window: every text token as a 4-bit pair (with alignment padding), then single plain rows */
  if (tiered || window) {
    cache_t t = make_cache(B, Hkv, G, T_cap, S_cap, window, 1);
    int32_t *row_src = xalloc((size_t)B * 2 * T * 4); uint8_t *row_tier = xalloc((size_t)B * 2 * T);
    int n_rows = 0;
    for (int tok = 0; tok < T; ++tok) {
      if (tiered && is_text[tok]) {
        if (n_rows % 2) { row_src[n_rows] = tok; row_tier[n_rows++] = 3; }
        row_src[n_rows] = tok; row_tier[n_rows++] = 1; row_src[n_rows] = tok; row_tier[n_rows++] = 2;
      } else { row_src[n_rows] = tok; row_tier[n_rows++] = 0; }
    }
    int32_t *rs = xalloc((size_t)B * n_rows * 4); uint8_t *rt = xalloc((size_t)B * n_rows);
    for (int b = 0; b < B; ++b) { memcpy(rs + (size_t)b * n_rows, row_src, (size_t)n_rows * 4); memcpy(rt + (size_t)b * n_rows, row_tier, n_rows); }
    orc_quantize_append_tiered(&t.c, k, v, T, rs, rt, n_rows, 0.8f, 1.0f, ORC_ROT_K | ORC_ROT_V, t.fine, t.k_win, t.v_win, window);
    t.c.T_len = n_rows;
    for (int step = 0; step < 3; ++step) {   /* plain single rows, identity mapping */
      orc_quantize_append_tiered(&t.c, k1, v1, first, NULL, NULL, first > 1 ? 1 : first, 0.8f, 1.0f, ORC_ROT_K | ORC_ROT_V, NULL,
                                 t.k_win, t.v_win, window);
      t.c.T_len += 1;
      if (first > 1) break;   /* n_src must equal n_rows for the identity mapping: only valid when first == 1 */
    }
    orc_decode_attention_tiered(&t.c, t.fine, t.k_win, t.v_win, window, Hq, q, 0.0884, ORC_ROT_Q | ORC_ROT_OUT, out, lse);
    for (int i = 0; i < B * Hq * 128; ++i) sum += out[i];
    orc_decode_attention_one_tiered(&t.c, t.fine, t.k_win, t.v_win, window, Hq, 0, 0, q, 0.0884, ORC_ROT_Q, out, lse);
    sum += out[5];
    free(row_src); free(row_tier); free(rs); free(rt); free_cache(&t);
  }
  free(k1); free(v1); free(k2); free(v2);
  free_cache(&a); free_cache(&p);
  free(k); free(v); free(qt); free(q); free(is_text); free(out); free(lse); free(mass);
  return sum;
}

int main(void) {
  double sum = 0.0;
  /* row-level functions */
  uint16_t row[128], ybf[128], sb[2]; int16_t z[2]; uint8_t codes[128];
  for (int rep = 0; rep < 64; ++rep) {
    for (int e = 0; e < 128; ++e) row[e] = rep == 0 ? 0 : (rep == 1 ? 0x7BFF : rand_half(rep == 2 ? 60000.0f : 3.0f));
    orc_quantize_row(row, rep % 2 ? 64 : 128, rep % 3 ? 0.8f : 1.0f, rep % 5 != 0, codes, sb, z, ybf);
    orc_quantize_row_bits(row, 128, 1.0f, 1, 4, codes, sb, z, ybf);
    sum += codes[3] + sb[0] + z[0] + orc_dequant(codes[7], sb[0], z[0]);
  }
  double H[16 * 16], x[16], y[16];
  orc_hadamard_dense(16, H);
  for (int i = 0; i < 16; ++i) x[i] = i;
  orc_wht_dense_f64(16, x, y);
  sum += H[17] + y[3];
  for (uint32_t h = 0; h < 65536; h += 257) sum += orc_float_to_bf16_rne(orc_half_to_float((uint16_t)h)) & 1;
  /* fold, massive activations, rotary embedding */
  {
    uint16_t *w = xalloc(256 * 128 * 2), *o = xalloc(256 * 128 * 2);
    for (int i = 0; i < 256 * 128; ++i) w[i] = rand_half(1.0f);
    orc_fold_hadamard(w, o, 256, 128, 1); orc_fold_hadamard(w, o, 256, 128, 0);
    sum += o[77]; free(w); free(o);
    cache_t m = make_cache(2, 3, 128, 128, 64, 0, 0);
    uint16_t *hid = xalloc(2 * 100 * 512 * 2); double *score = xalloc(2 * 100 * 8);
    for (int i = 0; i < 2 * 100 * 512; ++i) hid[i] = rand_half(i % 9001 == 0 ? 900.0f : 2.0f);
    orc_select_massive(&m.c, hid, 100, 512, 7, 100.0f, score); orc_select_massive(&m.c, hid, 100, 512, 64, 0.0f, NULL);
    sum += score[5] + m.c.sal_cnt[0]; free(hid); free(score); free_cache(&m);
    uint16_t *xr = xalloc(2 * 2 * 5 * 128 * 2), *orr = xalloc(2 * 2 * 5 * 128 * 2), *cs = xalloc(2 * 5 * 64 * 2), *sn = xalloc(2 * 5 * 64 * 2);
    for (int i = 0; i < 2 * 2 * 5 * 128; ++i) xr[i] = rand_half(2.0f);
    for (int i = 0; i < 2 * 5 * 64; ++i) { cs[i] = rand_half(1.0f); sn[i] = rand_half(1.0f); }
    orc_rope_rows(xr, orr, 2, 2, 5, cs, sn, 0); orc_rope_rows(xr, orr, 2, 2, 5, cs, sn, 5 * 64);
    sum += orr[9]; free(xr); free(orr); free(cs); free(sn);
  }
  /* the calls, shapes with ragged tails and both group sizes */
  sum += run_case(2, 4, 2, 128, 70, 16, 5, 0, 0);
  sum += run_case(1, 3, 3, 64, 33, 16, 40, 64, 1);     /* top_k above T: clamps */
  sum += run_case(2, 8, 1, 64, 131, 32, 9, 128, 1);
  sum += run_case(1, 2, 2, 128, 1, 1, 1, 64, 0);       /* a single row */
  if (!(sum == sum)) { printf("nan checksum\n"); return 1; }
  printf("ok %.6e\n", sum);
  return 0;
}

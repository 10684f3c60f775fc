/*
 * AKVQ-VL CPU oracle -- TEST INFRASTRUCTURE ONLY (see akvq_oracle.h).
 *
 * Build: gcc -O2 -ffp-contract=off -fno-fast-math -fopenmp -shared -fPIC
 * (contraction must stay off: the fp32 steps that decide a stored integer are specified as
 * individually rounded IEEE operations).
 *
 * Where the paper fixes the mathematics (Eq. 3-7, softmax attention) the code below is that
 * mathematics written out.  Where the paper is silent (rounding of each step, storage format,
 * tie rules) the choice made is marked "reading:" and is the same one the GPU library documents.
 */
#include "akvq_oracle.h"

#include <math.h>
#include <stdlib.h>
#include <string.h>

/* ------------------------------------------------------------------------------------------
 * binary16 / bfloat16 conversions, written out bit by bit.
 * pinned by: tests compare against numpy's float16 casts on every one of the 65536 patterns
 * and on random binary32 inputs.
 * ---------------------------------------------------------------------------------------- */
static float bits_to_float(uint32_t u) { float f; memcpy(&f, &u, 4); return f; }
static uint32_t float_to_bits(float f) { uint32_t u; memcpy(&u, &f, 4); return u; }

float orc_half_to_float(uint16_t h) {
  uint32_t sign = (uint32_t)(h >> 15) << 31;
  int exp = (h >> 10) & 0x1F;
  uint32_t man = h & 0x3FF;
  if (exp == 0x1F) return bits_to_float(sign | 0x7F800000u | (man << 13)); /* inf / nan */
  if (exp == 0) {
    /* zero or subnormal: value = man * 2^-24, exactly representable in binary32 */
    float v = (float)man * bits_to_float(0x33800000u); /* 2^-24 */
    return sign ? -v : v;
  }
  return bits_to_float(sign | ((uint32_t)(exp - 15 + 127) << 23) | (man << 13));
}

uint16_t orc_float_to_half_rne(float f) {
  uint32_t u = float_to_bits(f);
  uint16_t sign = (uint16_t)((u >> 16) & 0x8000);
  uint32_t a = u & 0x7FFFFFFFu;
  if (a >= 0x7F800000u) return (uint16_t)(sign | 0x7C00 | ((a > 0x7F800000u) ? 0x200 : 0)); /* inf / nan */
  if (a >= 0x477FF000u) return (uint16_t)(sign | 0x7C00); /* >= 65520 rounds to inf */
  if (a < 0x33000001u) return sign;                        /* <= 2^-25 rounds to zero (tie goes to even = 0) */
  int e = (int)(a >> 23) - 127;                            /* unbiased exponent */
  uint32_t m = (a & 0x7FFFFFu) | 0x800000u;                /* 24-bit significand */
  int shift = (e < -14) ? (13 + (-14 - e)) : 13;           /* bits to drop */
  uint32_t kept = m >> shift;
  uint32_t rem = m & ((1u << shift) - 1u);
  uint32_t halfway = 1u << (shift - 1);
  if (rem > halfway || (rem == halfway && (kept & 1u))) kept++;
  if (e < -14) return (uint16_t)(sign | kept);             /* subnormal (a carry lands on the smallest normal) */
  /* normal: kept has the implicit bit at position 10; a carry to bit 11 bumps the exponent through the add */
  return (uint16_t)(sign | (((uint32_t)(e + 15) << 10) + (kept - 0x400u)));
}

float orc_bf16_to_float(uint16_t b) { return bits_to_float((uint32_t)b << 16); }

uint16_t orc_float_to_bf16_rne(float f) {
  uint32_t u = float_to_bits(f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return (uint16_t)((u >> 16) | 0x40); /* quiet nan */
  uint32_t rem = u & 0xFFFFu, kept = u >> 16;
  if (rem > 0x8000u || (rem == 0x8000u && (kept & 1u))) kept++;
  return (uint16_t)kept;
}

/* ------------------------------------------------------------------------------------------
 * Walsh-Hadamard transform, Section III-C Eq. 7.
 * pinned by: H_2 and H_4 written out by hand from Eq. 7 (tests/golden/hadamard_small.txt);
 * H*H^T = I; H symmetric; butterfly == dense product; involution; Parseval; q.k preserved.
 * ---------------------------------------------------------------------------------------- */
void orc_hadamard_dense(int n, double *H) {
  /* H_1 = [1];  H_{2m} = 1/sqrt(2) * [[H_m, H_m], [H_m, -H_m]] */
  H[0] = 1.0;
  for (int m = 1; m < n; m *= 2) {
    /* grow the m x m block held in the top-left corner (row stride n) to 2m x 2m */
    for (int r = 0; r < m; ++r)
      for (int c = 0; c < m; ++c) {
        double v = H[(size_t)r * n + c] / sqrt(2.0);
        H[(size_t)r * n + c] = v;
        H[(size_t)r * n + (c + m)] = v;
        H[(size_t)(r + m) * n + c] = v;
        H[(size_t)(r + m) * n + (c + m)] = -v;
      }
  }
}

void orc_wht_dense_f64(int n, const double *x, double *y) {
  double *H = (double *)malloc(sizeof(double) * (size_t)n * n);
  orc_hadamard_dense(n, H);
  for (int c = 0; c < n; ++c) {
    double acc = 0.0;
    for (int r = 0; r < n; ++r) acc += x[r] * H[(size_t)r * n + c];
    y[c] = acc;
  }
  free(H);
}

/* reading: the rotation that decides stored integers is evaluated in binary32 as the fast transform
 * (Section III-C cites FWHT): stages with stride 1,2,4,...,64 in this order, each pair (a,b) replaced by
 * (a+b, a-b), every add individually rounded; the 2^-3.5 normalisation of Eq. 7 is applied afterwards. */
void orc_fwht128_f32(const float *x, float *u) {
  float buf[ORC_D];
  memcpy(buf, x, sizeof(buf));
  for (int h = 1; h < ORC_D; h *= 2)
    for (int base = 0; base < ORC_D; base += 2 * h)
      for (int i = base; i < base + h; ++i) {
        float a = buf[i], b = buf[i + h];
        buf[i] = a + b;
        buf[i + h] = a - b;
      }
  memcpy(u, buf, sizeof(buf));
}

/* ------------------------------------------------------------------------------------------
 * Quantizer, Section III-C Eq. 3-6 with n = 2 bits, per token, per group of G rotated channels.
 * pinned by: |y - y'| <= scale/2 (clip 1) and the clipped variant; codes monotone in y; the chosen code is
 * the nearest level (brute force over 0..3); a four-level group reproduces itself; constant group.
 * parity unpinned (paper silent, this build's readings): clip formula, fp16 storage of the scale and its
 * rounding direction, tie rule, order of the fp32 operations.
 * ---------------------------------------------------------------------------------------- */
#define ORC_INV_SQRT128_BITS 0x3DB504F3u /* 2^-3.5 rounded to binary32 */
#define ORC_ONE_THIRD_BITS 0x3EAAAAABu   /* 1/3 rounded to binary32 */
#define ORC_ONE_FIFTEENTH_BITS 0x3D888889u /* 1/15 rounded to binary32 */

static uint8_t round_clamp_code(double p, int zero, int top) {
  /* clamp( round_half_even(p + zero), 0, top ) evaluated exactly; p is an exact product of two binary32 numbers */
  if (!(p == p)) return 0;               /* nan: unspecified, keep it in range */
  if (p > 1.0e6) return (zero > -1000000) ? (uint8_t)top : 0;
  if (p < -1.0e6) return 0;
  double fl = floor(p);
  double frac = p - fl;                  /* exact */
  long k = (long)fl + (long)zero;
  if (frac > 0.5) k += 1;
  else if (frac == 0.5 && (k & 1L)) k += 1; /* tie -> even result */
  if (k < 0) k = 0;
  if (k > top) k = top;
  return (uint8_t)k;
}

void orc_quantize_row(const uint16_t *x_f16, int G, float clip, int rotate,
                      uint8_t *codes, uint16_t *scale_bits, int16_t *zero, uint16_t *y_bf16) {
  orc_quantize_row_bits(x_f16, G, clip, rotate, 2, codes, scale_bits, zero, y_bf16);
}

/* Eq. 3-6 with n = n_bits (2 or 4).  For 4 bits (the text tier of Section III-C.1) the same readings apply with
 * 2^n - 1 = 15; the stored scale saturates at 16376 so that four times it is still a binary16 number (the cache
 * stores a 4-bit row as two 2-bit rows, see orc_quantize_append_tiered). */
void orc_quantize_row_bits(const uint16_t *x_f16, int G, float clip, int rotate, int n_bits,
                           uint8_t *codes, uint16_t *scale_bits, int16_t *zero, uint16_t *y_bf16) {
  const int top = (1 << n_bits) - 1;
  const uint16_t s16_max = n_bits == 2 ? 0x7BFF : 0x73FF;
  float xf[ORC_D], u[ORC_D];
  for (int e = 0; e < ORC_D; ++e) xf[e] = orc_half_to_float(x_f16[e]);
  float kappa;
  if (rotate) {
    orc_fwht128_f32(xf, u);
    kappa = bits_to_float(ORC_INV_SQRT128_BITS);
  } else {
    memcpy(u, xf, sizeof(u));
    kappa = 1.0f;
  }
  /* the rotated row y = u * kappa; salient rows keep it as bfloat16 (Section III-C.1: salient tokens stay 16-bit).
   * reading: a zero is stored as +0.  The sign of a zero carries no information for attention, and an implementation
   * is free to hold intermediate butterfly values negated (b - a for a - b), which loses it. */
  for (int e = 0; e < ORC_D; ++e) {
    volatile float y = u[e] * kappa;
    if (y == 0.0f) y = 0.0f;
    y_bf16[e] = orc_float_to_bf16_rne(y);
  }
  const float third = bits_to_float(n_bits == 2 ? ORC_ONE_THIRD_BITS : ORC_ONE_FIFTEENTH_BITS);
  for (int g = 0; g < ORC_D / G; ++g) {
    float umin = u[g * G], umax = u[g * G];
    for (int e = g * G; e < (g + 1) * G; ++e) {
      if (u[e] < umin) umin = u[e];
      if (u[e] > umax) umax = u[e];
    }
    /* min/max of y equal the scaled min/max of u because rounding is monotone */
    volatile float gmin = umin * kappa, gmax = umax * kappa;
    /* reading: clipped_min = clip * min, clipped_max = clip * max */
    volatile float cmin = clip * gmin, cmax = clip * gmax;
    volatile float range = cmax - cmin;
    volatile float s32 = range * third;         /* Eq. 5: range / (2^n - 1) as a multiply by the rounded reciprocal */
    /* reading: the scale is stored as binary16, rounded UP so that the top level never falls below cmax */
    uint16_t s16;
    if (!(s32 > 0.0f)) s16 = 0x3C00;            /* constant group (or nan): scale 1 */
    else {
      s16 = orc_float_to_half_rne(s32);
      if (s16 > s16_max) s16 = s16_max;         /* saturate (65504 for 2 bits) */
      else if (orc_half_to_float(s16) < s32) s16 = (uint16_t)(s16 + 1);
      if (s16 > s16_max) s16 = s16_max;
    }
    float s = orc_half_to_float(s16);
    volatile float rcp = 1.0f / s;              /* all further arithmetic uses the stored scale */
    /* Eq. 6: zero = -round(cmin / scale) */
    volatile float zq = cmin * rcp;
    float zr = rintf(zq);                       /* round-half-even in the default rounding mode */
    long z = -(long)zr;
    if (zr != zr) z = 0;
    if (z > 32767) z = 32767;
    if (z < -32768) z = -32768;
    /* Eq. 3: X/scale evaluated as u * (kappa/scale); reading: the product is not rounded before the
     * round-to-integer, and the integer zero is added before rounding (changes ties only) */
    volatile float rcpu = rcp * kappa;
    for (int e = g * G; e < (g + 1) * G; ++e)
      codes[e] = round_clamp_code((double)u[e] * (double)rcpu, (int)z, top);
    scale_bits[g] = s16;
    zero[g] = (int16_t)z;
  }
}

double orc_dequant(uint8_t code, uint16_t scale_bits, int16_t zero) {
  /* Eq. 4: X' = scale * (Q(X) - zero) */
  return (double)orc_half_to_float(scale_bits) * ((double)code - (double)zero);
}

/* ------------------------------------------------------------------------------------------
 * Cache byte format (this build's own; parity of the format is a matter between the two
 * implementations, pinned by round trips and hand-computed positions).
 *
 * K plane of one (b,hkv): token blocks of 32; block = 64 chunks of 16 bytes (4 words).
 *   token t: blk=t/32, half=(t%32)/16, n=t%16.  channel e: m=e/32, j=(e%32)/8, i=e%8.
 *   chunk = 16*j + n; word in chunk = 2*half + m/2; code slot in word = 8*(m%2) + i; bit = 2*slot.
 * V plane of one (b,hkv): same block / chunk sizes, token-transposed.
 *   token t: blk=t/32, half=(t%32)/16, r=t%16, q=r/4, ii=r%4.  channel e: nb=e/16, n=e%16.
 *   chunk = 16*q + n; word in chunk = 2*(nb%2) + nb/4; bit = 16*half + 2*(4*((nb/2)%2) + ii).
 * V overlay plane: slot s: blk=s/32, half=(s%32)/16, r=s%16, q=r/4, ii=r%4; channel e: nb, n as above.
 *   uint16 index = blk*4096 + nb*512 + (16*q+n)*8 + 2*ii + half.
 * ---------------------------------------------------------------------------------------- */
void orc_k_code_pos(int t, int e, size_t *word, int *bit) {
  int blk = t / 32, half = (t % 32) / 16, n = t % 16;
  int m = e / 32, j = (e % 32) / 8, i = e % 8;
  *word = (size_t)blk * 256 + (size_t)(16 * j + n) * 4 + (size_t)(2 * half + m / 2);
  *bit = 2 * (8 * (m % 2) + i);
}

void orc_v_code_pos(int t, int e, size_t *word, int *bit) {
  int blk = t / 32, half = (t % 32) / 16, r = t % 16, q = r / 4, ii = r % 4;
  int nb = e / 16, n = e % 16;
  *word = (size_t)blk * 256 + (size_t)(16 * q + n) * 4 + (size_t)(2 * (nb % 2) + nb / 4);
  *bit = 16 * half + 2 * (4 * ((nb / 2) % 2) + ii);
}

size_t orc_vsal_pos(int slot, int e) {
  int blk = slot / 32, half = (slot % 32) / 16, r = slot % 16, q = r / 4, ii = r % 4;
  int nb = e / 16, n = e % 16;
  return (size_t)blk * 4096 + (size_t)nb * 512 + (size_t)(16 * q + n) * 8 + (size_t)(2 * ii + half);
}

static size_t plane_words(const orc_cache *c) { return (size_t)(c->T_cap / 32) * 256; }
static size_t bh_index(const orc_cache *c, int b, int h) { return (size_t)b * c->Hkv + h; }

uint8_t orc_get_code(const orc_cache *c, int tensor, int b, int h, int t, int e) {
  size_t w; int bit;
  if (tensor == 0) orc_k_code_pos(t, e, &w, &bit); else orc_v_code_pos(t, e, &w, &bit);
  const uint32_t *plane = (tensor == 0 ? c->k_codes : c->v_codes) + bh_index(c, b, h) * plane_words(c);
  return (uint8_t)((plane[w] >> bit) & 3u);
}

static void put_code(orc_cache *c, int tensor, int b, int h, int t, int e, uint8_t code) {
  size_t w; int bit;
  if (tensor == 0) orc_k_code_pos(t, e, &w, &bit); else orc_v_code_pos(t, e, &w, &bit);
  uint32_t *plane = (tensor == 0 ? c->k_codes : c->v_codes) + bh_index(c, b, h) * plane_words(c);
  plane[w] = (plane[w] & ~(3u << bit)) | ((uint32_t)code << bit);
}

static int valid_salient_count(const orc_cache *c, int b, int h) {
  int n = c->sal_cnt[bh_index(c, b, h)];
  if (n < 0) n = 0;
  if (n > c->S_cap) n = c->S_cap;
  return n;
}

/* rank of token t in the salient list of (b,h), or -1 */
static int salient_slot(const orc_cache *c, int b, int h, int t) {
  const int32_t *idx = c->sal_idx + bh_index(c, b, h) * c->S_cap;
  int n = valid_salient_count(c, b, h);
  for (int s = 0; s < n; ++s) if (idx[s] == t) return s;
  return -1;
}

/* ------------------------------------------------------------------------------------------
 * Salient-token selection, Section III-B.
 * TSA (III-B.1): every text token is salient.  pinned by: equals the index set of the mask (exact).
 * PSA (III-B.2): pivot tokens are the few that receive most of the attention (Section I); the score used is
 * the attention-column mass over the last W query rows; pinned by: sum of masses = W * (Hq/Hkv), a hand
 * case with W=1, full sort on small T, planted high-norm keys are selected.  parity unpinned: the score
 * itself replaces the paper's massive-activation detector, which needs a trained model.
 * ---------------------------------------------------------------------------------------- */
void orc_select_tsa(orc_cache *c, const uint8_t *is_text, int T) {
  for (int b = 0; b < c->B; ++b)
    for (int h = 0; h < c->Hkv; ++h) {
      int32_t *idx = c->sal_idx + bh_index(c, b, h) * c->S_cap;
      int n = 0;
      for (int t = 0; t < T; ++t)
        if (is_text[(size_t)b * T + t]) {
          if (n < c->S_cap) idx[n] = t;
          ++n;
        }
      c->sal_cnt[bh_index(c, b, h)] = n; /* true count; only the first S_cap positions are stored */
    }
}

typedef struct { double mass; int idx; } mass_item;
static int mass_cmp(const void *a, const void *b) {
  const mass_item *x = (const mass_item *)a, *y = (const mass_item *)b;
  if (x->mass > y->mass) return -1;
  if (x->mass < y->mass) return 1;
  return (x->idx > y->idx) - (x->idx < y->idx); /* equal mass: lower position first */
}
static int int_cmp(const void *a, const void *b) {
  int x = *(const int *)a, y = *(const int *)b;
  return (x > y) - (x < y);
}

static double bf16_round_of_half(uint16_t h) {
  /* reading: scoring uses bfloat16 operands (inputs arrive as binary16 and are rounded once) */
  return (double)orc_bf16_to_float(orc_float_to_bf16_rne(orc_half_to_float(h)));
}

/* top_k positions of one mass row (mass descending, then position ascending), written ascending to every list in
 * lists[0..n_lists) */
static void select_top_positions(const orc_cache *c, const double *mass, int T, int top_k, int32_t **lists,
                                 int32_t **counts, int n_lists) {
  mass_item *items = (mass_item *)malloc(sizeof(mass_item) * (size_t)T);
  for (int t = 0; t < T; ++t) { items[t].mass = mass[t]; items[t].idx = t; }
  qsort(items, (size_t)T, sizeof(mass_item), mass_cmp);
  int kk = top_k < T ? top_k : T;
  int *sel = (int *)malloc(sizeof(int) * (size_t)(kk > 0 ? kk : 1));
  for (int s = 0; s < kk; ++s) sel[s] = items[s].idx;
  qsort(sel, (size_t)kk, sizeof(int), int_cmp);
  for (int l = 0; l < n_lists; ++l) {
    for (int s = 0; s < kk && s < c->S_cap; ++s) lists[l][s] = sel[s];
    *counts[l] = kk;
  }
  free(sel); free(items);
}

/* share_heads != 0: the masses of the kv-heads of a batch element are added (head 0 first) and every head gets the
 * same list -- token-level pivots, as the paper has them (Section III-B.2: one pivot set per layer). */
static void select_psa_impl(orc_cache *c, int Hq, const uint16_t *q_tail, const uint16_t *k, int T, int W, int top_k,
                            double sm_scale, double *mass_out, int share_heads) {
  double *mass_all = (double *)malloc(sizeof(double) * (size_t)c->B * c->Hkv * T);
  const int r = Hq / c->Hkv;
  const int nbh = c->B * c->Hkv;
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < nbh; ++bh) {
    int b = bh / c->Hkv, h = bh % c->Hkv;
    double *mass = (double *)calloc((size_t)T, sizeof(double));
    double *kd = (double *)malloc(sizeof(double) * (size_t)T * ORC_D);
    double *logit = (double *)malloc(sizeof(double) * (size_t)T);
    const uint16_t *kp = k + ((size_t)bh * T) * ORC_D;
    for (size_t x = 0; x < (size_t)T * ORC_D; ++x) kd[x] = bf16_round_of_half(kp[x]);
    for (int hh = 0; hh < r; ++hh) {
      int hq = h * r + hh;
      for (int i = 0; i < W; ++i) {
        int pos = T - W + i;                     /* absolute position of this query row */
        const uint16_t *qp = q_tail + (((size_t)b * Hq + hq) * W + i) * ORC_D;
        double qd[ORC_D];
        for (int d = 0; d < ORC_D; ++d) qd[d] = bf16_round_of_half(qp[d]);
        double mx = -INFINITY;
        for (int t = 0; t <= pos; ++t) {          /* causal: keys up to and including the row's position */
          double acc = 0.0;
          for (int d = 0; d < ORC_D; ++d) acc += qd[d] * kd[(size_t)t * ORC_D + d];
          logit[t] = sm_scale * acc;
          if (logit[t] > mx) mx = logit[t];
        }
        double den = 0.0;
        for (int t = 0; t <= pos; ++t) den += exp(logit[t] - mx);
        for (int t = 0; t <= pos; ++t) mass[t] += exp(logit[t] - mx) / den;
      }
    }
    memcpy(mass_all + (size_t)bh * T, mass, sizeof(double) * (size_t)T);
    free(logit); free(kd); free(mass);
  }
  if (mass_out) memcpy(mass_out, mass_all, sizeof(double) * (size_t)c->B * c->Hkv * T);
  if (!share_heads) {
    for (int bh = 0; bh < nbh; ++bh) {
      int32_t *list = c->sal_idx + (size_t)bh * c->S_cap, *cnt = c->sal_cnt + bh;
      select_top_positions(c, mass_all + (size_t)bh * T, T, top_k, &list, &cnt, 1);
    }
  } else {
    double *sum = (double *)malloc(sizeof(double) * (size_t)T);
    int32_t **lists = (int32_t **)malloc(sizeof(int32_t *) * (size_t)c->Hkv);
    int32_t **cnts = (int32_t **)malloc(sizeof(int32_t *) * (size_t)c->Hkv);
    for (int b = 0; b < c->B; ++b) {
      for (int t = 0; t < T; ++t) sum[t] = 0.0;
      for (int h = 0; h < c->Hkv; ++h) {
        const double *m = mass_all + ((size_t)b * c->Hkv + h) * T;
        for (int t = 0; t < T; ++t) sum[t] += m[t];
        lists[h] = c->sal_idx + ((size_t)b * c->Hkv + h) * c->S_cap;
        cnts[h] = c->sal_cnt + ((size_t)b * c->Hkv + h);
      }
      select_top_positions(c, sum, T, top_k, lists, cnts, c->Hkv);
    }
    free(sum); free(lists); free(cnts);
  }
  free(mass_all);
}

void orc_select_psa(orc_cache *c, int Hq, const uint16_t *q_tail, const uint16_t *k, int T, int W, int top_k,
                    double sm_scale, double *mass_out) {
  select_psa_impl(c, Hq, q_tail, k, T, W, top_k, sm_scale, mass_out, 0);
}

void orc_select_psa_shared(orc_cache *c, int Hq, const uint16_t *q_tail, const uint16_t *k, int T, int W, int top_k,
                           double sm_scale, double *mass_out) {
  select_psa_impl(c, Hq, q_tail, k, T, W, top_k, sm_scale, mass_out, 1);
}

/* ------------------------------------------------------------------------------------------
 * Offline fold of the rotation into projection weights (Section III-C.2 / Fig. 7: H is merged into W_V and W_O so that
 * the value rotation and the output un-rotation cost nothing online).  w [rows][cols] binary16, row-major.
 *   axis 1: every aligned run of 128 columns of a row is rotated: out[r][128g..] = in[r][128g..] * H   (W_V, used as x*W_V)
 *   axis 0: every aligned run of 128 rows is rotated column-wise: out[128g..][c] = H * in[128g..][c]    (W_O, used as o*W_O)
 * Arithmetic as for cached rows: fp32 butterfly (stride 1..64), times 2^-3.5, rounded to binary16 (nearest even).
 * pinned by: equals the dense H product within binary16 rounding; folding twice returns the input within rounding;
 * (x*W_V)*H equals x*(W_V folded) within rounding.
 * ---------------------------------------------------------------------------------------- */
void orc_fold_hadamard(const uint16_t *w, uint16_t *out, int rows, int cols, int axis) {
  const float kappa = bits_to_float(ORC_INV_SQRT128_BITS);
  float x[ORC_D], u[ORC_D];
  if (axis == 1) {
    for (int r = 0; r < rows; ++r)
      for (int g = 0; g < cols / ORC_D; ++g) {
        for (int e = 0; e < ORC_D; ++e) x[e] = orc_half_to_float(w[(size_t)r * cols + g * ORC_D + e]);
        orc_fwht128_f32(x, u);
        for (int e = 0; e < ORC_D; ++e) {
          volatile float y = u[e] * kappa;
          out[(size_t)r * cols + g * ORC_D + e] = orc_float_to_half_rne(y);
        }
      }
  } else {
    for (int g = 0; g < rows / ORC_D; ++g)
      for (int c = 0; c < cols; ++c) {
        for (int e = 0; e < ORC_D; ++e) x[e] = orc_half_to_float(w[(size_t)(g * ORC_D + e) * cols + c]);
        orc_fwht128_f32(x, u);
        for (int e = 0; e < ORC_D; ++e) {
          volatile float y = u[e] * kappa;
          out[(size_t)(g * ORC_D + e) * cols + c] = orc_float_to_half_rne(y);
        }
      }
  }
}

/* ------------------------------------------------------------------------------------------
 * Pivot tokens from massive activations (Section III-B.2: tokens whose residual-stream activations are massive
 * attract the attention of the following layers; their indices are the pivot tokens).
 * reading (the paper gives neither a threshold nor a count rule; its ablation keeps 15 pivots): the score of a
 * token is the largest magnitude among its hidden-state channels; pivots are the top_k positions by score among
 * those whose score is at least `floor`; equal scores go to the lower position; the list is per batch element and
 * copied to every kv-head.  pinned by: planted activations are found; full sort; floor and tie cases.
 * parity unpinned by the paper (threshold, count).
 * ---------------------------------------------------------------------------------------- */
void orc_select_massive(orc_cache *c, const uint16_t *hidden, int T, int d_model, int top_k, float floor_,
                        double *score_out) {
  for (int b = 0; b < c->B; ++b) {
    mass_item *items = (mass_item *)malloc(sizeof(mass_item) * (size_t)T);
    int n = 0;
    for (int t = 0; t < T; ++t) {
      const uint16_t *row = hidden + ((size_t)b * T + t) * d_model;
      double mx = 0.0;
      for (int ch = 0; ch < d_model; ++ch) {
        double v = fabs((double)orc_half_to_float(row[ch]));
        if (v > mx) mx = v;
      }
      if (score_out) score_out[(size_t)b * T + t] = mx;
      if (mx >= (double)floor_ && mx > 0.0) { items[n].mass = mx; items[n].idx = t; ++n; }
    }
    qsort(items, (size_t)n, sizeof(mass_item), mass_cmp);
    int kk = top_k < n ? top_k : n;
    int *sel = (int *)malloc(sizeof(int) * (size_t)(kk > 0 ? kk : 1));
    for (int s_ = 0; s_ < kk; ++s_) sel[s_] = items[s_].idx;
    qsort(sel, (size_t)kk, sizeof(int), int_cmp);
    for (int h = 0; h < c->Hkv; ++h) {
      int32_t *idx = c->sal_idx + bh_index(c, b, h) * c->S_cap;
      for (int s_ = 0; s_ < kk && s_ < c->S_cap; ++s_) idx[s_] = sel[s_];
      c->sal_cnt[bh_index(c, b, h)] = kk;
    }
    free(sel); free(items);
  }
}

/* ----------------------------------------------------------------------------------------
 * Rotary position embedding in front of the rotation (Section III-C.2, Fig. 6: Q and K are rotated by H after RoPE).
 * Convention of the LLaMA family the paper evaluates (RoFormer, Su et al. 2021, in its "rotate half" form): channel i
 * pairs with channel i + 64, angle pos * theta_i:
 *     out[i]      = x[i] * cos_i - x[i + 64] * sin_i
 *     out[i + 64] = x[i + 64] * cos_i + x[i] * sin_i
 * The caller supplies cos and sin as binary16 tables (what an fp16 model holds), one row of 64 per position.
 * reading (the paper does not state the arithmetic): both products of binary16 numbers are exact in binary32; their
 * sum or difference is rounded once to binary32 and then to binary16, the format in which the model hands K and q
 * on.  Evaluated here in double (exact for these operands up to the one rounding that follows).
 * x, out: [B][H][n][128]; cos, sin: [n][64], batch b at b * batch_stride (0: one table for every batch entry).
 * ---------------------------------------------------------------------------------------- */
void orc_rope_rows(const uint16_t *x, uint16_t *out, int B, int H, int n, const uint16_t *cos_t, const uint16_t *sin_t,
                   long batch_stride) {
  for (int b = 0; b < B; ++b)
    for (int h = 0; h < H; ++h)
      for (int r = 0; r < n; ++r) {
        const uint16_t *xr = x + (((size_t)b * H + h) * n + r) * ORC_D;
        uint16_t *o = out + (((size_t)b * H + h) * n + r) * ORC_D;
        const uint16_t *cr = cos_t + (size_t)b * batch_stride + (size_t)r * 64;
        const uint16_t *sr = sin_t + (size_t)b * batch_stride + (size_t)r * 64;
        for (int i = 0; i < 64; ++i) {
          const double lo = orc_half_to_float(xr[i]), hi = orc_half_to_float(xr[i + 64]);
          const double c = orc_half_to_float(cr[i]), sn = orc_half_to_float(sr[i]);
          const float a = (float)(lo * c - hi * sn);
          const float bb = (float)(hi * c + lo * sn);
          o[i] = orc_float_to_half_rne(a);
          o[i + 64] = orc_float_to_half_rne(bb);
        }
      }
}

/* ------------------------------------------------------------------------------------------
 * Write path: rotate, quantize (Eq. 3-6), pack; salient rows also keep a bfloat16 copy.
 * Every row gets 2-bit codes and meta; a row listed in sal_idx additionally gets an overlay row at the
 * slot equal to its rank in the list, and bit 15 of its meta words is set.
 * ---------------------------------------------------------------------------------------- */
void orc_quantize_append(orc_cache *c, const uint16_t *k_new, const uint16_t *v_new, int n_new, float clip,
                         int rot) {
  const int ng = ORC_D / c->G;
  const int nbh = c->B * c->Hkv;
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < nbh; ++bh) {
    int b = bh / c->Hkv, h = bh % c->Hkv;
    for (int i = 0; i < n_new; ++i) {
      int t = c->T_len + i;
      int slot = salient_slot(c, b, h, t);
      for (int tensor = 0; tensor < 2; ++tensor) {
        const uint16_t *row = (tensor == 0 ? k_new : v_new) + ((size_t)bh * n_new + i) * ORC_D;
        uint8_t codes[ORC_D]; uint16_t sb[2]; int16_t z[2]; uint16_t ybf[ORC_D];
        orc_quantize_row(row, c->G, clip, (rot & (tensor == 0 ? ORC_ROT_K : ORC_ROT_V)) != 0, codes, sb, z, ybf);
        for (int e = 0; e < ORC_D; ++e) put_code(c, tensor, b, h, t, e, codes[e]);
        uint32_t *meta = (tensor == 0 ? c->k_meta : c->v_meta) + ((size_t)bh * c->T_cap + t) * ng;
        for (int g = 0; g < ng; ++g)
          meta[g] = (uint32_t)sb[g] | (slot >= 0 ? 0x8000u : 0u) | ((uint32_t)(uint16_t)z[g] << 16);
        if (slot >= 0) {
          if (tensor == 0) {
            uint16_t *dst = c->k_sal + ((size_t)bh * c->S_cap + slot) * ORC_D;
            memcpy(dst, ybf, sizeof(ybf));
          } else {
            uint16_t *plane = c->v_sal + (size_t)bh * c->S_cap * ORC_D;
            for (int e = 0; e < ORC_D; ++e) plane[orc_vsal_pos(slot, e)] = ybf[e];
          }
        }
      }
    }
  }
}

/* ------------------------------------------------------------------------------------------
 * Tiered write path (Section III-C.1: text tokens 4-bit, the rest 2-bit).  Cache row T_len + r of batch element b
 * takes source token row_src[b][r] and tier row_tier[b][r]:
 *   0  plain 2-bit row (as orc_quantize_append, overlay included when the row is listed in sal_idx);
 *   1  coarse half of a 4-bit token, 2  its fine half (always the next row; the pair starts on an even row):
 *      the token is quantized to 4 bits (scale s, zero z4, code c4), then stored as two 2-bit rows
 *        coarse: codes c4 >> 2, scale 4*s, zero z4 >> 2 (floor);   fine: codes c4 & 3, scale s, zero z4 & 3
 *      so that  4*s*(hi - zc) + s*(lo - zf) = s*(c4 - z4)  exactly;
 *   3  padding row: meta = salient bit with scale bits 0 (a marker no real row has), so decode ignores it.
 * fine_mask [B][T_cap/32]: bit (t % 32) of word t/32 is set for fine halves, cleared for every other written row.
 * reading (the paper gives no storage format): this pairing is this build's own; parity unpinned by the paper,
 * pinned by the identity above and by attention over directly dequantized 4-bit values.
 * ---------------------------------------------------------------------------------------- */
void orc_quantize_append_tiered(orc_cache *c, const uint16_t *k_src, const uint16_t *v_src, int n_src,
                                const int32_t *row_src, const uint8_t *row_tier, int n_rows, float clip2,
                                float clip4, int rot, uint32_t *fine_mask, uint16_t *k_win, uint16_t *v_win,
                                int W) {
  const int ng = ORC_D / c->G;
  const int nbh = c->B * c->Hkv;
  const int t_end = c->T_len + n_rows;
  if (fine_mask)
  for (int b = 0; b < c->B; ++b)
    for (int i = 0; i < n_rows; ++i) {
      int t = c->T_len + i;
      uint32_t *w = fine_mask + (size_t)b * (c->T_cap / 32) + t / 32;
      if (row_tier[(size_t)b * n_rows + i] == 2) *w |= 1u << (t % 32); else *w &= ~(1u << (t % 32));
    }
#pragma omp parallel for schedule(dynamic)
  for (int bh = 0; bh < nbh; ++bh) {
    int b = bh / c->Hkv, h = bh % c->Hkv;
    for (int i = 0; i < n_rows; ++i) {
      int t = c->T_len + i;
      int tier = row_tier ? row_tier[(size_t)b * n_rows + i] : 0;
      int src = row_src ? row_src[(size_t)b * n_rows + i] : i;
      int slot = tier == 0 ? salient_slot(c, b, h, t) : -1;
      /* recent window (Section III-B.1 keeps the most recent tokens 16-bit): the last W of the appended rows also go
       * to ring slot t % W as bfloat16 (rotated), overwriting the row that leaves the window -- whose codes were
       * written when it was appended, so leaving the window needs no work.  Fine halves and padding rows carry no
       * token: their slots are zeroed. */
      const int in_win = (W > 0) && (t >= t_end - W);
      for (int tensor = 0; tensor < 2; ++tensor) {
        uint32_t *meta = (tensor == 0 ? c->k_meta : c->v_meta) + ((size_t)bh * c->T_cap + t) * ng;
        if (in_win && (tier == 2 || tier == 3)) {
          if (tensor == 0) memset(k_win + ((size_t)bh * W + t % W) * ORC_D, 0, sizeof(uint16_t) * ORC_D);
          else for (int e = 0; e < ORC_D; ++e) v_win[(size_t)bh * W * ORC_D + orc_vsal_pos(t % W, e)] = 0;
        }
        if (tier == 3) {
          for (int e = 0; e < ORC_D; ++e) put_code(c, tensor, b, h, t, e, 0);
          for (int g = 0; g < ng; ++g) meta[g] = 0x8000u; /* scale bits 0 + salient bit: the padding marker */
          continue;
        }
        const uint16_t *row = (tensor == 0 ? k_src : v_src) + ((size_t)bh * n_src + src) * ORC_D;
        uint8_t codes[ORC_D]; uint16_t sb[2]; int16_t z[2]; uint16_t ybf[ORC_D];
        const int rotate = (rot & (tensor == 0 ? ORC_ROT_K : ORC_ROT_V)) != 0;
        if (in_win && tier != 2) { /* ybf does not depend on the bit width */
          uint16_t yb[ORC_D]; uint8_t cc[ORC_D]; uint16_t s2[2]; int16_t z2[2];
          orc_quantize_row_bits(row, c->G, clip2, rotate, 2, cc, s2, z2, yb);
          if (tensor == 0) memcpy(k_win + ((size_t)bh * W + t % W) * ORC_D, yb, sizeof(yb));
          else for (int e = 0; e < ORC_D; ++e) v_win[(size_t)bh * W * ORC_D + orc_vsal_pos(t % W, e)] = yb[e];
        }
        if (tier == 0) {
          orc_quantize_row_bits(row, c->G, clip2, rotate, 2, codes, sb, z, ybf);
          for (int e = 0; e < ORC_D; ++e) put_code(c, tensor, b, h, t, e, codes[e]);
          for (int g = 0; g < ng; ++g)
            meta[g] = (uint32_t)sb[g] | (slot >= 0 ? 0x8000u : 0u) | ((uint32_t)(uint16_t)z[g] << 16);
          if (slot >= 0) {
            if (tensor == 0) memcpy(c->k_sal + ((size_t)bh * c->S_cap + slot) * ORC_D, ybf, sizeof(ybf));
            else {
              uint16_t *plane = c->v_sal + (size_t)bh * c->S_cap * ORC_D;
              for (int e = 0; e < ORC_D; ++e) plane[orc_vsal_pos(slot, e)] = ybf[e];
            }
          }
        } else {
          orc_quantize_row_bits(row, c->G, clip4, rotate, 4, codes, sb, z, ybf);
          for (int e = 0; e < ORC_D; ++e)
            put_code(c, tensor, b, h, t, e, tier == 1 ? (uint8_t)(codes[e] >> 2) : (uint8_t)(codes[e] & 3));
          for (int g = 0; g < ng; ++g) {
            uint16_t s_row = sb[g];
            int z_row;
            if (tier == 1) {
              s_row = orc_float_to_half_rne(4.0f * orc_half_to_float(sb[g])); /* exact: sb <= 16376 */
              z_row = (z[g] >= 0) ? (z[g] >> 2) : -((-(int)z[g] + 3) >> 2);  /* floor(z4 / 4) */
            } else {
              z_row = (int)z[g] - 4 * ((z[g] >= 0) ? (z[g] >> 2) : -((-(int)z[g] + 3) >> 2)); /* z4 mod 4 in 0..3 */
            }
            meta[g] = (uint32_t)s_row | ((uint32_t)(uint16_t)(int16_t)z_row << 16);
          }
        }
      }
    }
  }
}

/* ------------------------------------------------------------------------------------------
 * Read path: softmax attention of one decode query over the cached rows (Section II-A, Eq. 2 context),
 * using the dequantized (Eq. 4) or bfloat16 rows, all in fp64, dense, two-pass softmax.
 * The query is rotated with the dense H_128 (Section III-C: rotate Q and K after RoPE); the output is
 * rotated back (H is its own inverse); rot selects which of the two happen (ORC_ROT_Q | ORC_ROT_OUT is the method).
 * pinned by: a numpy brute-force attention over independently dequantized rows; T=1; equal scores give
 * the mean; shift invariance; an all-salient cache matches attention over the original K,V up to
 * bfloat16 rounding; GQA equals MHA with repeated KV heads.
 * ---------------------------------------------------------------------------------------- */
static void cached_row(const orc_cache *c, int tensor, int b, int h, int t, int slot, double *row) {
  size_t bh = bh_index(c, b, h);
  if (slot >= 0) {
    if (tensor == 0) {
      const uint16_t *src = c->k_sal + (bh * c->S_cap + slot) * ORC_D;
      for (int e = 0; e < ORC_D; ++e) row[e] = (double)orc_bf16_to_float(src[e]);
    } else {
      const uint16_t *plane = c->v_sal + bh * c->S_cap * ORC_D;
      for (int e = 0; e < ORC_D; ++e) row[e] = (double)orc_bf16_to_float(plane[orc_vsal_pos(slot, e)]);
    }
    return;
  }
  const int ng = ORC_D / c->G;
  const uint32_t *meta = (tensor == 0 ? c->k_meta : c->v_meta) + (bh * c->T_cap + t) * ng;
  for (int e = 0; e < ORC_D; ++e) {
    uint32_t mw = meta[e / c->G];
    row[e] = orc_dequant(orc_get_code(c, tensor, b, h, t, e), (uint16_t)(mw & 0x7FFFu), (int16_t)(mw >> 16));
  }
}

void orc_decode_attention_one(const orc_cache *c, int Hq, int b, int hq, const uint16_t *q_row, double sm_scale,
                              int rot, double *out, double *lse) {
  orc_decode_attention_one_tiered(c, NULL, NULL, NULL, 0, Hq, b, hq, q_row, sm_scale, rot, out, lse);
}

/* first row of the recent window: the last W rows, the boundary moved up to an even row so that a (coarse, fine)
 * pair is never split (the window then holds W or W-1 rows) */
static int window_start(int T_len, int W) {
  if (W <= 0) return T_len;
  int t = T_len - W;
  if (t < 0) t = 0;
  return (t + 1) & ~1;
}
static void window_row(const uint16_t *k_win, const uint16_t *v_win, int W, size_t bh, int tensor, int t, double *row) {
  int slot = t % W;
  if (tensor == 0) {
    const uint16_t *src = k_win + (bh * W + slot) * ORC_D;
    for (int e = 0; e < ORC_D; ++e) row[e] = (double)orc_bf16_to_float(src[e]);
  } else {
    const uint16_t *plane = v_win + bh * W * ORC_D;
    for (int e = 0; e < ORC_D; ++e) row[e] = (double)orc_bf16_to_float(plane[orc_vsal_pos(slot, e)]);
  }
}

/* fine_mask (may be NULL): rows flagged there are the fine halves of 4-bit tokens; such a row and the row before
 * it are one token whose value is the sum of the two dequantized rows (Eq. 4 applied to each half). */
void orc_decode_attention_one_tiered(const orc_cache *c, const uint32_t *fine_mask, const uint16_t *k_win,
                                     const uint16_t *v_win, int W, int Hq, int b, int hq, const uint16_t *q_row,
                                     double sm_scale, int rot, double *out, double *lse) {
  const int r = Hq / c->Hkv;
  const int h = hq / r;
  const int T = c->T_len;
  double qd[ORC_D], qrot[ORC_D];
  for (int d = 0; d < ORC_D; ++d) qd[d] = (double)orc_half_to_float(q_row[d]);
  if (rot & ORC_ROT_Q) orc_wht_dense_f64(ORC_D, qd, qrot);
  else memcpy(qrot, qd, sizeof(qrot));
  int *slot_of = (int *)malloc(sizeof(int) * (size_t)T);
  for (int t = 0; t < T; ++t) slot_of[t] = -1;
  {
    const int32_t *idx = c->sal_idx + bh_index(c, b, h) * c->S_cap;
    int n = valid_salient_count(c, b, h);
    for (int s = 0; s < n; ++s) if (idx[s] >= 0 && idx[s] < T) slot_of[idx[s]] = s;
  }
  double *score = (double *)malloc(sizeof(double) * (size_t)T);
  double row[ORC_D], row2[ORC_D];
  double mx = -INFINITY;
  const uint32_t *fm = fine_mask ? fine_mask + (size_t)b * (c->T_cap / 32) : NULL;
  const int t_win = window_start(T, (k_win && v_win) ? W : 0);
#define ORC_IS_FINE(t) (fm && ((fm[(t) / 32] >> ((t) % 32)) & 1u))
  /* a token = one row, or a (coarse, fine) pair of rows; skipped rows: fine halves (counted with their coarse row)
   * and rows flagged salient that have no overlay slot (padding) */
  for (int t = 0; t < T; ++t) {
    score[t] = -INFINITY;
    if (ORC_IS_FINE(t)) continue;
    const uint32_t mk = c->k_meta[(bh_index(c, b, h) * c->T_cap + t) * (ORC_D / c->G)];
    if (t >= t_win) { /* recent window: the 16-bit ring row is the token, whatever its tier */
      if ((mk & 0xFFFFu) == 0x8000u) continue; /* padding row */
      window_row(k_win, v_win, W, bh_index(c, b, h), 0, t, row);
    } else {
      if (slot_of[t] < 0 && (mk & 0x8000u)) continue;
      cached_row(c, 0, b, h, t, slot_of[t], row);
      if (t + 1 < T && ORC_IS_FINE(t + 1)) {
        cached_row(c, 0, b, h, t + 1, -1, row2);
        for (int e = 0; e < ORC_D; ++e) row[e] += row2[e];
      }
    }
    double acc = 0.0;
    for (int e = 0; e < ORC_D; ++e) acc += qrot[e] * row[e];
    score[t] = sm_scale * acc;
    if (score[t] > mx) mx = score[t];
  }
  double den = 0.0;
  for (int t = 0; t < T; ++t) if (score[t] != -INFINITY) den += exp(score[t] - mx);
  double orot[ORC_D];
  for (int e = 0; e < ORC_D; ++e) orot[e] = 0.0;
  for (int t = 0; t < T; ++t) {
    if (score[t] == -INFINITY) continue;
    double p = exp(score[t] - mx) / den;
    if (t >= t_win) {
      window_row(k_win, v_win, W, bh_index(c, b, h), 1, t, row);
    } else {
      cached_row(c, 1, b, h, t, slot_of[t], row);
      if (t + 1 < T && ORC_IS_FINE(t + 1)) {
        cached_row(c, 1, b, h, t + 1, -1, row2);
        for (int e = 0; e < ORC_D; ++e) row[e] += row2[e];
      }
    }
    for (int e = 0; e < ORC_D; ++e) orot[e] += p * row[e];
  }
#undef ORC_IS_FINE
  if (rot & ORC_ROT_OUT) orc_wht_dense_f64(ORC_D, orot, out);
  else memcpy(out, orot, sizeof(orot));
  if (lse) *lse = mx + log(den);
  free(score); free(slot_of);
}

void orc_decode_attention(const orc_cache *c, int Hq, const uint16_t *q, double sm_scale, int rot,
                          double *out, double *lse) {
  orc_decode_attention_tiered(c, NULL, NULL, NULL, 0, Hq, q, sm_scale, rot, out, lse);
}

void orc_decode_attention_tiered(const orc_cache *c, const uint32_t *fine_mask, const uint16_t *k_win,
                                 const uint16_t *v_win, int W, int Hq, const uint16_t *q, double sm_scale,
                                 int rot, double *out, double *lse) {
  const int n = c->B * Hq;
#pragma omp parallel for schedule(dynamic)
  for (int x = 0; x < n; ++x) {
    int b = x / Hq, hq = x % Hq;
    orc_decode_attention_one_tiered(c, fine_mask, k_win, v_win, W, Hq, b, hq, q + (size_t)x * ORC_D, sm_scale, rot,
                                    out + (size_t)x * ORC_D, lse ? lse + x : NULL);
  }
}

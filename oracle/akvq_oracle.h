/*
 * AKVQ-VL CPU oracle -- TEST INFRASTRUCTURE ONLY.
 *
 * A plain, slow, single-purpose CPU implementation of what the AKVQ-VL KV-cache hot
 * path computes (arXiv 2501.15021: Section III-B salient-token identification,
 * Section III-C Eq. 3-7 quantizer and Walsh-Hadamard rotation, Section II-A Eq. 2
 * decode attention).  It exists so that the GPU library can be checked against
 * something that can be read next to the paper.  Only the tests, the smoke check and
 * the benchmark's cpu_baseline leg may call it; the product path never does.
 *
 * It shares no code, header, table or constant generator with the HIP library.
 * The cache byte format below is re-stated here from its written definition.
 *
 * Parity status of each function is stated in its comment ("pinned by ..." /
 * "parity unpinned").
 */
#ifndef AKVQ_ORACLE_H
#define AKVQ_ORACLE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

enum { ORC_D = 128, ORC_TB = 32 };

/* Host-memory mirror of one layer's mixed-precision cache (all pointers are host memory).
 *   k_codes/v_codes : [B][Hkv][T_cap/32][256] uint32 words, 2-bit codes (layout: see orc_k_code_pos / orc_v_code_pos)
 *   k_meta/v_meta   : [B][Hkv][T_cap][D/G] uint32: bits 0-14 fp16 scale, bit 15 salient flag, bits 16-31 int16 zero
 *   k_sal           : [B][Hkv][S_cap][128] bf16 bit patterns, rotated rows, natural channel order
 *   v_sal           : [B][Hkv][S_cap/32][4096] bf16 bit patterns, rotated rows, tiled (see orc_vsal_pos)
 *   sal_idx         : [B][Hkv][S_cap] ascending token positions; sal_cnt : [B][Hkv]
 */
typedef struct {
  int32_t B, Hkv, G, T_cap, S_cap, T_len;
  uint32_t *k_codes, *v_codes;
  uint32_t *k_meta, *v_meta;
  uint16_t *k_sal, *v_sal;
  int32_t *sal_idx, *sal_cnt;
} orc_cache;

/* ---- scalar format helpers (IEEE binary16 / bfloat16 <-> binary32, round-to-nearest-even) ---- */
float orc_half_to_float(uint16_t h);
uint16_t orc_float_to_half_rne(float f);
float orc_bf16_to_float(uint16_t b);
uint16_t orc_float_to_bf16_rne(float f);

/* ---- Walsh-Hadamard (Section III-C, Eq. 7) ---- */
/* Dense orthonormal H_n built by the Sylvester recursion of Eq. 7 (n a power of two), row-major, fp64. */
void orc_hadamard_dense(int n, double *H);
/* y = x * H_n with the dense matrix (the definition), fp64. */
void orc_wht_dense_f64(int n, const double *x, double *y);
/* Un-normalised 128-point butterfly in fp32: 7 stages, stride 1,2,...,64, each (a,b)->(a+b,a-b). */
void orc_fwht128_f32(const float *x, float *u);

/* ---- quantizer (Section III-C, Eq. 3-6) for one head vector ---- */
/* x_f16: 128 binary16 bit patterns.  rotate!=0: rotate by H_128 first.  Outputs: codes[128] in 0..3 (natural rotated
 * channel order), scale_bits[D/G], zero[D/G], y_bf16[128] (rotated row as bfloat16).  Two bits. */
void orc_quantize_row(const uint16_t *x_f16, int G, float clip, int rotate,
                      uint8_t *codes, uint16_t *scale_bits, int16_t *zero, uint16_t *y_bf16);
/* The same with n_bits = 2 or 4 (codes in 0..2^n-1); 4 bits is the text tier of Section III-C.1. */
void orc_quantize_row_bits(const uint16_t *x_f16, int G, float clip, int rotate, int n_bits,
                           uint8_t *codes, uint16_t *scale_bits, int16_t *zero, uint16_t *y_bf16);
/* Dequantized value of Eq. 4 in fp64 from stored fields. */
double orc_dequant(uint8_t code, uint16_t scale_bits, int16_t zero);

/* ---- cache byte format (this build's own; not from the paper) ---- */
void orc_k_code_pos(int t, int e, size_t *word, int *bit); /* word index inside one (b,hkv) plane, bit offset */
void orc_v_code_pos(int t, int e, size_t *word, int *bit);
size_t orc_vsal_pos(int slot, int e);                      /* uint16 index inside one (b,hkv) v_sal plane */
uint8_t orc_get_code(const orc_cache *c, int tensor /*0=K,1=V*/, int b, int h, int t, int e);

/* ---- the three calls of the hot path ---- */
/* TSA (Section III-B.1): salient = text positions.  is_text [B][T].  Writes the cache's sal_idx / sal_cnt. */
void orc_select_tsa(orc_cache *c, const uint8_t *is_text, int T);
/* PSA (Section III-B.2, with attention-column mass as the pivot score).  q_tail [B][Hq][W][128], k [B][Hkv][T][128],
 * both binary16, un-rotated.  mass_out (optional) [B][Hkv][T] fp64.  Writes sal_idx / sal_cnt. */
void orc_select_psa(orc_cache *c, int Hq, const uint16_t *q_tail, const uint16_t *k, int T, int W, int top_k,
                    double sm_scale, double *mass_out);
/* The same with token-level pivots (Section III-B.2: one pivot set per layer): the masses of a batch element's kv-heads
 * are added and every kv-head gets the same list.  mass_out stays per kv-head. */
void orc_select_psa_shared(orc_cache *c, int Hq, const uint16_t *q_tail, const uint16_t *k, int T, int W, int top_k,
                           double sm_scale, double *mass_out);
/* Offline fold of H_128 into a projection matrix w [rows][cols] binary16 (Section III-C.2, Fig. 7): axis 1 rotates every
 * aligned run of 128 columns of each row (W_V), axis 0 every aligned run of 128 rows column-wise (W_O). */
void orc_fold_hadamard(const uint16_t *w, uint16_t *out, int rows, int cols, int axis);
/* Pivots from massive activations (Section III-B.2): hidden [B][T][d_model] binary16 (a block's residual-stream output);
 * score = max |channel| per token; the top_k positions with score >= floor (ties -> lower position), the same list for
 * every kv-head.  score_out (optional) [B][T] fp64.  Writes sal_idx / sal_cnt. */
void orc_select_massive(orc_cache *c, const uint16_t *hidden, int T, int d_model, int top_k, float floor_,
                        double *score_out);
/* Rotary position embedding ("rotate half" pairing, channel i with i + 64) of rows x [B][H][n][128] binary16 with
 * binary16 tables cos, sin [n][64] (batch b at b * batch_stride; 0 = shared); result rounded to binary16.  Runs in front
 * of the write path (on K) and of decode (on q) when the caller hands over pre-RoPE tensors (Section III-C.2, Fig. 6). */
void orc_rope_rows(const uint16_t *x, uint16_t *out, int B, int H, int n, const uint16_t *cos_t, const uint16_t *sin_t,
                   long batch_stride);
/* Which rotations a call applies.  The method is ORC_ROT_K | ORC_ROT_V on the write path and ORC_ROT_Q | ORC_ROT_OUT on
 * the read path; a cleared bit means the tensor is already in (or stays in) the rotated domain -- the offline fold of
 * Section III-C.2 clears ORC_ROT_V and ORC_ROT_OUT; all four cleared is plain round-to-nearest quantization without the
 * rotation (the ablation baseline of Table III). */
enum { ORC_ROT_K = 1, ORC_ROT_V = 2, ORC_ROT_Q = 1, ORC_ROT_OUT = 2 };
/* Write path: rows [T_len, T_len+n_new) of K and V ([B][Hkv][n_new][128] binary16).  Does not change T_len. */
void orc_quantize_append(orc_cache *c, const uint16_t *k_new, const uint16_t *v_new, int n_new, float clip,
                         int rot);
/* Tiered write path: cache row T_len + r of batch b takes source token row_src[b][r] (index into k_src / v_src,
 * [B][Hkv][n_src][128]) with tier row_tier[b][r]: 0 = 2-bit, 1 / 2 = coarse / fine half of a 4-bit token (two 2-bit
 * rows), 3 = padding.  fine_mask [B][T_cap/32] marks the fine halves.  Does not change T_len. */
void orc_quantize_append_tiered(orc_cache *c, const uint16_t *k_src, const uint16_t *v_src, int n_src,
                                const int32_t *row_src, const uint8_t *row_tier, int n_rows, float clip2,
                                float clip4, int rot, uint32_t *fine_mask, uint16_t *k_win, uint16_t *v_win,
                                int W);
/* row_src / row_tier / fine_mask may be NULL (plain rows, identity mapping).  Recent window (W > 0): k_win
 * [B][Hkv][W][128] and v_win [B][Hkv][W/32][4096] (tiled like v_sal) bfloat16 rings, zero-initialised by the caller;
 * the last W appended rows are also written to slot t % W.  Decode then reads rows t >= window start from the ring. */
/* Read path: decode attention (Eq. 2 with the dequantized cache), fp64.  q [B][Hq][128] binary16.
 * out [B][Hq][128]; lse (optional) [B][Hq].  rot & ORC_ROT_Q: q is rotated first; rot & ORC_ROT_OUT: out = o~ * H_128. */
void orc_decode_attention(const orc_cache *c, int Hq, const uint16_t *q, double sm_scale, int rot,
                          double *out, double *lse);
/* One (b,hq) output only -- used to spot-check full-size runs. */
void orc_decode_attention_one(const orc_cache *c, int Hq, int b, int hq, const uint16_t *q_row, double sm_scale,
                              int rot, double *out, double *lse);

/* The same over a cache with 4-bit tokens stored as row pairs (fine_mask may be NULL: no such tokens). */
void orc_decode_attention_tiered(const orc_cache *c, const uint32_t *fine_mask, const uint16_t *k_win,
                                 const uint16_t *v_win, int W, int Hq, const uint16_t *q, double sm_scale,
                                 int rot, double *out, double *lse);
void orc_decode_attention_one_tiered(const orc_cache *c, const uint32_t *fine_mask, const uint16_t *k_win,
                                     const uint16_t *v_win, int W, int Hq, int b, int hq, const uint16_t *q_row,
                                     double sm_scale, int rot, double *out, double *lse);

#ifdef __cplusplus
}
#endif
#endif

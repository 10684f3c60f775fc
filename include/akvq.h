/*
 * akvq.h -- C ABI of the AKVQ-VL KV-cache hot path for AMD MI355X (gfx950).
 *
 * Method: arXiv 2501.15021 (AKVQ-VL).  Salient tokens (text tokens in Text-Salient-Attention layers,
 * pivot tokens in Pivot-Token-Salient-Attention layers, Section III-B) stay 16-bit; every other cached
 * Key/Value row is rotated by the 128-point Walsh-Hadamard matrix (Section III-C.2, Eq. 7) and stored as
 * group-wise asymmetric 2-bit codes (Section III-C.1, Eq. 3-6).  Decode attention reads that cache directly.
 *
 * Conventions
 *   - Every pointer named "device" is GPU memory owned by the caller.  The library allocates nothing,
 *     frees nothing and never synchronises: each call validates its arguments on the host, enqueues
 *     kernels on `stream` (a hipStream_t passed as void*, NULL = default stream) and returns.
 *   - All device pointers must be 16-byte aligned, except is_text (bytes, any alignment).
 *   - B * Hkv (and B * Hq for the pivot score) must not exceed 65535 (a launch-grid limit): AKVQ_ERR_UNSUPPORTED.
 *   - Return value: AKVQ_OK or a negative akvq_status.  Argument errors launch nothing.
 *   - head_dim is fixed to 128, codes are 2-bit, the quantization group G is 64 or 128 channels of
 *     the rotated head vector.
 *
 * Cache format (one layer; this library's own, MFMA-operand-native)
 *   Tokens are stored in blocks of 32.  One block of one (batch, kv-head) plane is 1024 bytes =
 *   64 chunks of 16 bytes (4 little-endian uint32 words); a 64-lane wavefront loads a block with one
 *   128-bit load per lane and finds its matrix-core operand in its own registers.
 *   k_codes [B][Hkv][T_cap/32][256 words]
 *       token t: blk=t/32, half=(t%32)/16, n=t%16.  rotated channel e: m=e/32, j=(e%32)/8, i=e%8.
 *       word = blk*256 + (16*j+n)*4 + 2*half + m/2;  bits [2s, 2s+2) with s = 8*(m%2) + i.
 *   v_codes [B][Hkv][T_cap/32][256 words]   (token-transposed inside the block)
 *       token t: blk, half as above, r=t%16, q=r/4, ii=r%4.  channel e: nb=e/16, n=e%16.
 *       word = blk*256 + (16*q+n)*4 + 2*(nb%2) + nb/4;  bits [16*half + 2p, +2) with p = 4*((nb/2)%2) + ii.
 *   k_meta, v_meta [B][Hkv][T_cap][128/G] uint32
 *       bits 0-14 scale (IEEE binary16, positive), bit 15 = row is salient (its 2-bit copy is ignored
 *       by decode), bits 16-31 zero-point (int16).  Dequantized value = scale * (code - zero)  (Eq. 4).
 *   k_sal [B][Hkv][S_cap][128] bfloat16: rotated salient rows, natural channel order (round to nearest even of the
 *       fp32 value; a zero is stored as +0).
 *   v_sal [B][Hkv][S_cap/32][4096] bfloat16: rotated salient rows, tiled: slot s: blk=s/32,
 *       half=(s%32)/16, r=s%16, q=r/4, ii=r%4; channel e: nb=e/16, n=e%16;
 *       index = blk*4096 + nb*512 + (16*q+n)*8 + 2*ii + half.
 *   sal_idx [B][Hkv][S_cap] int32 ascending token positions; sal_cnt [B][Hkv] int32 (values above S_cap
 *       mean "S_cap stored, more were found"; consumers clamp).
 *   T_cap and S_cap must be multiples of 64.
 */
#ifndef AKVQ_H
#define AKVQ_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  AKVQ_OK = 0,
  AKVQ_ERR_INVALID_ARG = -1, /* null / misaligned pointer, non-positive size, Hq not a multiple of Hkv, W > T ... */
  AKVQ_ERR_UNSUPPORTED = -2, /* G not in {64,128}, Hq/Hkv > 8, W not a multiple of 16 ... */
  AKVQ_ERR_CAPACITY = -3,    /* T_len + n_new > T_cap, top_k > S_cap */
  AKVQ_ERR_WORKSPACE = -4,   /* workspace smaller than akvq_*_workspace_bytes() */
  AKVQ_ERR_HIP = -5          /* a kernel launch failed; see akvq_last_hip_error() */
} akvq_status;

enum { AKVQ_MODE_TSA = 0, AKVQ_MODE_PSA = 1, AKVQ_MODE_PSA_SHARED = 2 };

/* flags */
enum {
  AKVQ_V_PREROTATED = 1u, /* quantize_append: V rows arrive already rotated (H folded into W_V offline,
                             Section III-C.2 / Fig. 7); skip the transform on V */
  AKVQ_OUT_ROTATED = 2u,  /* decode_attention: leave the output in the rotated domain (H folded into W_O) */
  AKVQ_K_PREROTATED = 4u, /* quantize_append: K rows arrive already rotated; skip the transform on K */
  AKVQ_Q_PREROTATED = 8u, /* decode_attention: q arrives already rotated; skip the transform on q.
                             All four together make the library transform nothing: with inputs that were never
                             rotated this is plain round-to-nearest quantization, the ablation baseline of Table III */
  AKVQ_OUT_FP16 = 16u     /* decode_attention: out is [B][Hq][128] binary16 (the fp32 result rounded to nearest even)
                             instead of fp32 */
};

/* Tier of a cache row written by akvq_quantize_append_tiered (Section III-C.1: text tokens 4-bit, the rest 2-bit).
 * A 4-bit token occupies two consecutive cache rows, the first on an even row: its 4-bit code c4, scale s and
 * zero-point z4 are stored as a coarse 2-bit row (codes c4 >> 2, scale 4*s, zero floor(z4/4)) and a fine 2-bit row
 * (codes c4 & 3, scale s, zero z4 mod 4), so that the two dequantized rows add up to s*(c4 - z4) exactly. */
enum { AKVQ_TIER_2BIT = 0, AKVQ_TIER_4BIT_COARSE = 1, AKVQ_TIER_4BIT_FINE = 2, AKVQ_TIER_PAD = 3 };

/* Recent window (Section III-B.1: the most recent tokens stay 16-bit).  Two bfloat16 rings owned by the caller and
 * zero-initialised before the first append: k_win [B][Hkv][W][128] (row-major), v_win [B][Hkv][W/32][4096] (tiled like
 * v_sal).  Cache row t lives in slot t % W while it is among the last W rows; every row also gets its codes when it is
 * appended, so a row that leaves the window needs no work ("quantize on evict" is free: the quantizer is per token).
 * The window starts at the even row at or above T_len - W, so a 4-bit pair is never split.  W is a multiple of 64. */
typedef struct akvq_window {
  uint16_t *k_win, *v_win; /* device */
  int32_t W;
} akvq_window;

/* Rotary position embedding applied by the library in front of the rotation (Section III-C.2, Fig. 6: Q and K are
 * rotated by H after RoPE), for callers that hand over pre-RoPE K rows / queries and save the separate pass.
 * Pairing of the LLaMA family ("rotate half"): out[i] = x[i]*cos_i - x[i+64]*sin_i, out[i+64] = x[i+64]*cos_i +
 * x[i]*sin_i, i < 64.  cos / sin: device, binary16 (the tables an fp16 model holds), one row of 64 per position, 16-byte
 * aligned; batch element b reads its rows at b * batch_stride elements (0: one table for every batch element; else a
 * multiple of 8).  Arithmetic: the two products are exact in fp32, their sum is rounded once to fp32 and then to
 * binary16 (the format a separate RoPE pass would have stored); the rotation then starts from those binary16 values. */
typedef struct akvq_rope {
  const uint16_t *cos, *sin; /* device */
  int64_t batch_stride;
} akvq_rope;

/* One layer's cache.  Plain data; every pointer is device memory owned by the caller (layout above).
 * T_len is the number of valid rows; the caller advances it after akvq_quantize_append. */
typedef struct akvq_cache {
  int32_t B, Hkv, G, T_cap, S_cap, T_len;
  uint32_t *k_codes, *v_codes; /* device */
  uint32_t *k_meta, *v_meta;   /* device */
  uint16_t *k_sal, *v_sal;     /* device */
  int32_t *sal_idx, *sal_cnt;  /* device */
} akvq_cache;

const char *akvq_strerror(int status);
int akvq_last_hip_error(void); /* hipError_t of the most recent failed launch in this thread, 0 if none */
int akvq_version(void);

/* Host helper: byte sizes of the eight device arrays of a cache with the given shape fields
 * (order: k_codes, v_codes, k_meta, v_meta, k_sal, v_sal, sal_idx, sal_cnt).  Returns AKVQ_OK or an error. */
int akvq_cache_bytes(const akvq_cache *shape, size_t out_bytes[8]);

/* Host helpers: device workspace each call needs (bytes; 0 on invalid arguments). */
size_t akvq_select_workspace_bytes(int B, int Hq, int Hkv, int T, int W);
size_t akvq_decode_workspace_bytes(int B, int Hq, int n_split);
/* Host helper: number of KV splits akvq_decode_attention uses when n_split <= 0 is passed. */
int akvq_decode_default_splits(int B, int Hkv, int T_len);

/* Host helper: how the decode kernels deal the n_tiles tiles of the code stream (64 rows each when Hq == Hkv, else 32)
 * to n_split KV splits: split `split` reads tiles [*begin, *end) (equal runs of ceil(n_tiles / n_split); trailing
 * splits can be empty).  Returns the split whose run holds the last tile, which in akvq_decode_step is the one that
 * writes the new row (0 when n_tiles is 0), or AKVQ_ERR_INVALID_ARG. */
int akvq_decode_split_range(int n_tiles, int n_split, int split, int *begin, int *end);

/*
 * akvq_select_salient -- Section III-B: write the salient-token list of every (batch, kv-head).
 *   mode AKVQ_MODE_TSA (III-B.1): salient = text positions.  Needs is_text (device, [B][T] uint8).
 *   mode AKVQ_MODE_PSA (III-B.2): salient = the top_k positions by attention-column mass
 *       mass[b][hkv][t] = sum over the Hq/Hkv query heads of the group and the W last prompt rows i of
 *       softmax_t( sm_scale * q_i . k_t )[t], row i sitting at position T-W+i and seeing keys t <= T-W+i.
 *       Operands are rounded to bfloat16, products accumulate in fp32 on the matrix cores, softmax in fp32.
 *       Needs q_tail (device, [B][Hq][W][128] binary16, post-RoPE) and k (device, [B][Hkv][T][128] binary16,
 *       post-RoPE, un-rotated).  Ties go to the lower position.  W must be a multiple of 16, W <= T, W <= 64.
 *   mode AKVQ_MODE_PSA_SHARED: token-level pivots as in the paper (one pivot set per layer): the masses of a batch
 *       element's kv-heads are added (head order, fp32) and every kv-head gets the top_k positions of the sum.
 *   Output: c->sal_idx (ascending) and c->sal_cnt.  mass_out (device, [B][Hkv][T] fp32) is optional (PSA).
 *   workspace: device, akvq_select_workspace_bytes() bytes (PSA only; may be NULL for TSA).
 */
int akvq_select_salient(const akvq_cache *c, int mode, const uint8_t *is_text, const void *q_tail, int Hq,
                        const void *k, int T, int W, int top_k, float sm_scale, float *mass_out,
                        void *workspace, size_t workspace_bytes, void *stream);

/*
 * akvq_fold_hadamard -- offline mode of Section III-C.2 (Fig. 7): fold H_128 into a projection matrix once, so that
 *   values arrive rotated (AKVQ_V_PREROTATED) and the rotated attention output (AKVQ_OUT_ROTATED) is consumed as is.
 *   w_in, w_out: device, [rows][cols] binary16, row-major (w_out may equal w_in only for axis 1).
 *   axis 1: every aligned run of 128 columns of each row becomes run * H_128   (W_V used as x * W_V; cols % 128 == 0);
 *   axis 0: every aligned run of 128 rows becomes H_128 * run, column by column (W_O used as o * W_O; rows % 128 == 0).
 *   fp32 butterfly (strides 1..64), times 2^-3.5, rounded to binary16.
 */
int akvq_fold_hadamard(const void *w_in, void *w_out, int rows, int cols, int axis, void *stream);

/*
 * akvq_select_massive -- Section III-B.2 as the paper states it: pivot tokens are the tokens whose residual-stream
 *   activations are massive.  hidden: device, [B][T][d_model] binary16 (a Transformer block's output), d_model a
 *   multiple of 512.  score[b][t] = max over channels of |hidden|; the salient list of every kv-head of batch element b
 *   is the top_k positions by score among those with score >= floor (and > 0), equal scores to the lower position,
 *   ascending.  c->sal_cnt receives the number kept (<= top_k).  score_out: optional device [B][T] fp32.
 *   workspace: device, akvq_massive_workspace_bytes(B, T) bytes.
 */
size_t akvq_massive_workspace_bytes(int B, int T);
int akvq_select_massive(const akvq_cache *c, const void *hidden, int T, int d_model, int top_k, float floor,
                        float *score_out, void *workspace, size_t workspace_bytes, void *stream);

/*
 * akvq_quantize_append -- Section III-C write path for rows [T_len, T_len + n_new).
 *   k_new, v_new: device, [B][Hkv][n_new][128] binary16 (K post-RoPE, un-rotated).
 *   Each row is rotated (fp32 butterfly, stride 1..64, then 2^-3.5), its groups get scale / zero-point
 *   (Eq. 5-6 with clipped_min = clip*min, clipped_max = clip*max; scale stored as binary16 rounded up) and
 *   2-bit codes (Eq. 3, round-half-even of x/scale + zero).  Rows listed in c->sal_idx additionally get a
 *   bfloat16 copy in the overlay at the slot equal to their rank in the list, and the salient bit in meta.
 *   c->sal_idx / c->sal_cnt must already be final for these rows.  Does not modify c->T_len.
 */
int akvq_quantize_append(const akvq_cache *c, const void *k_new, const void *v_new, int n_new, float clip,
                         uint32_t flags, void *stream);

/*
 * akvq_decode_attention -- read path: out[b][hq] = softmax_t( sm_scale * q~ . k^_t ) v^_t over the T_len cached rows
 *   (Section II-A decode step with the Section III-C cache), q~ = q * H_128, k^/v^ = bfloat16 overlay row if the
 *   row is salient else scale*(code - zero).  Split over T (n_split partial softmaxes merged exactly);
 *   fp32 accumulation.  Output is rotated back by H_128 unless AKVQ_OUT_ROTATED.
 *   q: device [B][Hq][128] binary16.  out: device [B][Hq][128] fp32 (binary16 with AKVQ_OUT_FP16).  lse_out: optional
 *   device [B][Hq] fp32.
 *   n_split <= 0 picks akvq_decode_default_splits().  workspace: device, akvq_decode_workspace_bytes() bytes.
 */
int akvq_decode_attention(const akvq_cache *c, const void *q, int Hq, float sm_scale, void *out, float *lse_out,
                          int n_split, void *workspace, size_t workspace_bytes, uint32_t flags, void *stream);

/*
 * akvq_decode_attention_static -- akvq_decode_attention for callers that cannot allocate or pass device scratch memory:
 *   code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  The split-KV partial results
 *   go to a fixed array inside the library's device image (akvq_decode_static_scratch_bytes() = 8 MiB per GPU, held
 *   until the process ends) instead of a caller workspace; the call allocates and frees nothing.  Same kernels, same
 *   results as akvq_decode_attention with the same n_split.  Requests whose partials do not fit
 *   (akvq_decode_workspace_bytes(B, Hq, n_split) above the limit, i.e. B * Hq * n_split > 15887) are rejected with
 *   AKVQ_ERR_WORKSPACE before anything is launched.  Every call on a GPU shares that GPU's array: calls that overlap
 *   on one GPU (different streams, or threads) race; calls on one stream are ordered.  Nothing in the array needs to
 *   start at zero: every (head, split) slot is written by the call before its merge pass reads it.
 */
size_t akvq_decode_static_scratch_bytes(void);
int akvq_decode_attention_static(const akvq_cache *c, const void *q, int Hq, float sm_scale, void *out, float *lse_out,
                                 int n_split, uint32_t flags, void *stream);

/*
 * akvq_quantize_append_tiered -- the write path with the 4-bit text tier of Section III-C.1.
 *   Cache row T_len + r of batch element b takes source token row_src[b][r] (an index into k_src / v_src, device,
 *   [B][Hkv][n_src][128] binary16) and tier row_tier[b][r] (device, [B][n_rows] uint8, AKVQ_TIER_*):
 *     2BIT         as akvq_quantize_append with clip2 (overlay and salient bit if the row is listed in c->sal_idx);
 *     4BIT_COARSE  / 4BIT_FINE: the two halves of one token quantized to 4 bits (Eq. 3-6 with 15 levels, clip4, scale
 *                  stored as binary16 rounded up and at most 16376); the pair must start on an even cache row, both
 *                  rows name the same source token, and neither may be listed in c->sal_idx;
 *     PAD          a row decode ignores (used to align a pair); its meta is 0x8000 (salient bit, scale bits 0).
 *   row_src, row_tier and fine_mask may all be NULL: plain rows with the identity mapping (n_rows = n_src).
 *   win (may be NULL): the last W of the appended rows are also written to the recent-window rings.
 *   fine_mask: device, [B][T_cap/32] uint32, zero-initialised by the caller before the first append; bit t%32 of word
 *   t/32 is set for fine halves and cleared for every other row written here.
 *   row_src entries are clamped to [0, n_src); other violations of the rules above give unspecified values, no fault.
 *   Does not modify c->T_len (advance it by n_rows).
 */
int akvq_quantize_append_tiered(const akvq_cache *c, const void *k_src, const void *v_src, int n_src,
                                const int32_t *row_src, const uint8_t *row_tier, int n_rows, float clip2,
                                float clip4, uint32_t *fine_mask, const akvq_window *win, uint32_t flags,
                                void *stream);

/*
 * akvq_decode_attention_tiered -- akvq_decode_attention over a cache that holds 4-bit tokens as row pairs:
 *   a row flagged in fine_mask and the row before it are one token (their scores add up before the softmax, the
 *   token is counted once, both rows take its weight).  win (may be NULL): rows from the window start on are read
 *   from the 16-bit rings instead of their codes.  fine_mask and win NULL = akvq_decode_attention.
 */
int akvq_decode_attention_tiered(const akvq_cache *c, const uint32_t *fine_mask, const akvq_window *win,
                                 const void *q, int Hq, float sm_scale, void *out, float *lse_out, int n_split,
                                 void *workspace, size_t workspace_bytes, uint32_t flags, void *stream);

/*
 * akvq_quantize_append_rope / akvq_decode_attention_rope -- the tiered entry points with the rotary position embedding
 *   fused in front of the rotation (Section III-C.2, Fig. 6).  k_src holds pre-RoPE rows; source token s of batch
 *   element b uses table row s (rope->cos/sin hold n_src rows per batch element).  q holds pre-RoPE queries; batch
 *   element b uses table row 0 of its table (one position per decode step).  V and everything else as in the tiered
 *   entry points; rope == NULL makes them identical to those.  AKVQ_K_PREROTATED / AKVQ_Q_PREROTATED cannot be
 *   combined with a table (the embedding precedes the rotation): AKVQ_ERR_INVALID_ARG.
 */
int akvq_quantize_append_rope(const akvq_cache *c, const void *k_src, const void *v_src, int n_src,
                              const int32_t *row_src, const uint8_t *row_tier, int n_rows, float clip2, float clip4,
                              uint32_t *fine_mask, const akvq_window *win, const akvq_rope *rope, uint32_t flags,
                              void *stream);
int akvq_decode_attention_rope(const akvq_cache *c, const uint32_t *fine_mask, const akvq_window *win, const void *q,
                               const akvq_rope *rope, int Hq, float sm_scale, void *out, float *lse_out, int n_split,
                               void *workspace, size_t workspace_bytes, uint32_t flags, void *stream);

/*
 * akvq_decode_step -- one generated token in one launch: the new token's K and V rows (k_new, v_new: device,
 *   [B][Hkv][1][128] binary16) are written to cache row T_len exactly as akvq_quantize_append_rope would write a single
 *   plain row (codes, meta, the recent-window rings, the overlay if the row is listed in c->sal_idx), then decode
 *   attention runs over the T_len + 1 rows as akvq_decode_attention_rope would: the cache holds the bits of the
 *   separate append, the output those of the separate decode call when n_split is 1 (with more splits the 16-bit rows
 *   are all read by one split, so they enter the sums in another order).  The new row is written by the workgroups
 *   of the KV split that holds the row's tile (akvq_decode_split_range) before they read it; no other workgroup
 *   reads it.
 *   c->T_len is the number of rows already cached (0 is allowed); advance it by one
 *   afterwards.  rope (may be NULL): one table row per batch element, used for the new K row and for q.  clip: the
 *   2-bit clip ratio.  flags: write- and read-path flags together.  Everything else as in the two entry points.
 */
int akvq_decode_step(const akvq_cache *c, const uint32_t *fine_mask, const akvq_window *win, const void *k_new,
                     const void *v_new, const void *q, const akvq_rope *rope, int Hq, float clip, float sm_scale,
                     void *out, float *lse_out, int n_split, void *workspace, size_t workspace_bytes, uint32_t flags,
                     void *stream);

/*
 * akvq_stream_read -- measurement aid, no part of the method: one pass of plain 128-bit loads over src (device, 16-byte
 *   aligned, `bytes` a multiple of 16), nothing computed but an exclusive-or, nothing stored (sink: device, one
 *   uint32, written only if the data happen to fold to a magic value).  non_temporal != 0: the loads carry the
 *   non-temporal hint, as the decode kernels' loads of the cache stream do.  Its rate is the practical streaming-read
 *   ceiling of the GPU to hold the cache kernels against, beside the published HBM peak.
 */
int akvq_stream_read(const void *src, size_t bytes, uint32_t *sink, int non_temporal, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* AKVQ_H */

// C ABI of libakvq (declared in include/akvq.h): argument validation, size helpers, kernel dispatch.
// Nothing here allocates, frees or synchronises; every call enqueues on the caller's stream and returns.
#include "../../include/akvq.h"

#include <hip/hip_runtime.h>

#include "akvq_kernels.h"

namespace {

thread_local int g_last_hip_error = 0;

inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }
inline size_t round_up(size_t x, size_t a) { return (x + a - 1) / a * a; }

int check_cache_shape(const akvq_cache *c) {
  if (!c) return AKVQ_ERR_INVALID_ARG;
  if (c->B <= 0 || c->Hkv <= 0 || c->T_cap <= 0 || c->S_cap <= 0 || c->T_len < 0) return AKVQ_ERR_INVALID_ARG;
  if (c->G != 64 && c->G != 128) return AKVQ_ERR_UNSUPPORTED;
  if (c->T_cap % 64 != 0 || c->S_cap % 64 != 0) return AKVQ_ERR_INVALID_ARG;
  if (c->T_len > c->T_cap) return AKVQ_ERR_CAPACITY;
  return AKVQ_OK;
}

int check_cache_pointers(const akvq_cache *c) {
  const void *p[8] = {c->k_codes, c->v_codes, c->k_meta, c->v_meta, c->k_sal, c->v_sal, c->sal_idx, c->sal_cnt};
  for (const void *x : p)
    if (!x || !aligned16(x)) return AKVQ_ERR_INVALID_ARG;
  return AKVQ_OK;
}

// (batch, head) units index the second grid dimension of the streaming kernels, which the runtime caps at 65535
constexpr long kMaxGridUnits = 65535;
inline bool too_many_units(long units) { return units > kMaxGridUnits; }

int hip_status(hipError_t e) {
  if (e == hipSuccess) return AKVQ_OK;
  g_last_hip_error = (int)e;
  return AKVQ_ERR_HIP;
}

}  // namespace

extern "C" {

const char *akvq_strerror(int status) {
  switch (status) {
    case AKVQ_OK: return "ok";
    case AKVQ_ERR_INVALID_ARG: return "invalid argument";
    case AKVQ_ERR_UNSUPPORTED: return "unsupported configuration";
    case AKVQ_ERR_CAPACITY: return "capacity exceeded";
    case AKVQ_ERR_WORKSPACE: return "workspace too small";
    case AKVQ_ERR_HIP: return "HIP launch failed";
    default: return "unknown status";
  }
}

int akvq_last_hip_error(void) { return g_last_hip_error; }

int akvq_version(void) { return 100; }

int akvq_cache_bytes(const akvq_cache *shape, size_t out_bytes[8]) {
  int st = check_cache_shape(shape);
  if (st != AKVQ_OK) return st;
  if (!out_bytes) return AKVQ_ERR_INVALID_ARG;
  const size_t bh = (size_t)shape->B * shape->Hkv;
  const size_t codes = bh * (size_t)(shape->T_cap / 32) * 1024;
  const size_t meta = bh * (size_t)shape->T_cap * (128 / shape->G) * 4;
  const size_t sal = bh * (size_t)shape->S_cap * 128 * 2;
  out_bytes[0] = codes; out_bytes[1] = codes;
  out_bytes[2] = meta;  out_bytes[3] = meta;
  out_bytes[4] = sal;   out_bytes[5] = sal;
  out_bytes[6] = bh * (size_t)shape->S_cap * 4;
  out_bytes[7] = round_up(bh * 4, 16);
  return AKVQ_OK;
}

static int select_chunks(int T) { return (int)(((long)T + akvq::kScoreChunk - 1) / akvq::kScoreChunk); }

size_t akvq_select_workspace_bytes(int B, int Hq, int Hkv, int T, int W) {
  if (B <= 0 || Hq <= 0 || Hkv <= 0 || T <= 0 || W <= 0) return 0;
  const size_t stats = (size_t)B * Hq * select_chunks(T) * W * 2 * sizeof(float);
  const size_t mass = (size_t)B * Hkv * T * sizeof(float);
  const size_t shared = (size_t)B * T * sizeof(float);  // AKVQ_MODE_PSA_SHARED: the kv-heads' masses added
  return round_up(stats, 256) + round_up(mass, 256) + round_up(shared, 256);
}

size_t akvq_decode_workspace_bytes(int B, int Hq, int n_split) {
  if (B <= 0 || Hq <= 0 || n_split <= 0) return 0;
  return round_up((size_t)B * Hq * n_split * akvq::kPartialStride * sizeof(float), 256);
}

int akvq_decode_default_splits(int B, int Hkv, int T_len) {
  if (B <= 0 || Hkv <= 0 || T_len <= 0) return 1;
  const long units = (long)B * Hkv;            // one workgroup of four wavefronts per (unit, split)
  if (units >= 512) return 1;                  // already two workgroups per CU: finish in one kernel, no merge pass
  const int tiles = (T_len + 63) / 64;
  long want = (512 + units - 1) / units;       // two workgroups per CU; more splits only add merge work
  long cap = tiles / 16 > 1 ? tiles / 16 : 1;  // keep at least four 64-token tiles per wavefront
  if (want > cap) want = cap;
  if (want > 64) want = 64;
  if (want < 1) want = 1;
  // A split adds the merge launch (about 8 us end to end): with more than 128 units it only pays when every workgroup
  // still streams at least 48 tiles (measured: 256 units of 64 tiles run 19.7 us unsplit, 21.7 us in two splits).
  if (units > 128 && tiles / want < 48) want = tiles / 48 > 1 ? tiles / 48 : 1;
  return (int)want;
}

int akvq_decode_split_range(int n_tiles, int n_split, int split, int *begin, int *end) {
  if (n_tiles < 0 || n_split <= 0 || split < 0 || split >= n_split || !begin || !end) return AKVQ_ERR_INVALID_ARG;
  akvq::decode_split_range(n_tiles, n_split, split, *begin, *end);
  return akvq::decode_last_tile_split(n_tiles, n_split);
}

int akvq_select_salient(const akvq_cache *c, int mode, const uint8_t *is_text, const void *q_tail, int Hq,
                        const void *k, int T, int W, int top_k, float sm_scale, float *mass_out,
                        void *workspace, size_t workspace_bytes, void *stream) {
  int st = check_cache_shape(c);
  if (st != AKVQ_OK) return st;
  if (!c->sal_idx || !c->sal_cnt || !aligned16(c->sal_idx) || !aligned16(c->sal_cnt)) return AKVQ_ERR_INVALID_ARG;
  if (T <= 0 || T > c->T_cap) return AKVQ_ERR_INVALID_ARG;
  akvq::SelectArgs a{};
  a.sal_idx = c->sal_idx; a.sal_cnt = c->sal_cnt;
  a.B = c->B; a.Hkv = c->Hkv; a.T = T; a.S_cap = c->S_cap;
  hipStream_t s = static_cast<hipStream_t>(stream);
  if (mode == AKVQ_MODE_TSA) {
    if (!is_text) return AKVQ_ERR_INVALID_ARG;
    a.is_text = is_text;
    a.Hq = c->Hkv;
    return hip_status(akvq::launch_select_tsa(a, s));
  }
  if (mode != AKVQ_MODE_PSA && mode != AKVQ_MODE_PSA_SHARED) return AKVQ_ERR_INVALID_ARG;
  if (!q_tail || !k || !aligned16(q_tail) || !aligned16(k)) return AKVQ_ERR_INVALID_ARG;
  if (Hq <= 0 || Hq % c->Hkv != 0 || W <= 0 || W > T || top_k <= 0) return AKVQ_ERR_INVALID_ARG;
  if (W % 16 != 0 || W > 64) return AKVQ_ERR_UNSUPPORTED;
  if (too_many_units((long)c->B * Hq)) return AKVQ_ERR_UNSUPPORTED;
  if (top_k > c->S_cap) return AKVQ_ERR_CAPACITY;
  if (mass_out && !aligned16(mass_out)) return AKVQ_ERR_INVALID_ARG;
  if (!workspace || !aligned16(workspace)) return AKVQ_ERR_INVALID_ARG;
  if (workspace_bytes < akvq_select_workspace_bytes(c->B, Hq, c->Hkv, T, W)) return AKVQ_ERR_WORKSPACE;
  a.q_tail = static_cast<const uint16_t *>(q_tail);
  a.k = static_cast<const uint16_t *>(k);
  a.Hq = Hq; a.W = W; a.top_k = top_k; a.sm_scale = sm_scale;
  a.n_chunk = select_chunks(T);
  a.row_stats = static_cast<float *>(workspace);
  const size_t stats = round_up((size_t)c->B * Hq * a.n_chunk * W * 2 * sizeof(float), 256);
  const size_t mass_bytes = round_up((size_t)c->B * c->Hkv * T * sizeof(float), 256);
  a.mass = mass_out ? mass_out : reinterpret_cast<float *>(static_cast<char *>(workspace) + stats);
  if (mode == AKVQ_MODE_PSA_SHARED)
    a.mass_shared = reinterpret_cast<float *>(static_cast<char *>(workspace) + stats + mass_bytes);
  return hip_status(akvq::launch_select_psa(a, s));
}

int akvq_fold_hadamard(const void *w_in, void *w_out, int rows, int cols, int axis, void *stream) {
  if (!w_in || !w_out || !aligned16(w_in) || !aligned16(w_out) || rows <= 0 || cols <= 0) return AKVQ_ERR_INVALID_ARG;
  if (axis != 0 && axis != 1) return AKVQ_ERR_INVALID_ARG;
  if ((axis == 1 ? cols : rows) % 128 != 0) return AKVQ_ERR_INVALID_ARG;
  if (axis == 0 && w_in == w_out) return AKVQ_ERR_INVALID_ARG;
  if (axis == 0 && too_many_units(rows / 128)) return AKVQ_ERR_UNSUPPORTED;
  return hip_status(akvq::launch_fold_hadamard(static_cast<const uint16_t *>(w_in), static_cast<uint16_t *>(w_out), rows,
                                               cols, axis, static_cast<hipStream_t>(stream)));
}

int akvq_stream_read(const void *src, size_t bytes, uint32_t *sink, int non_temporal, void *stream) {
  if (!src || !sink || !aligned16(src) || bytes < 16 || bytes % 16 != 0) return AKVQ_ERR_INVALID_ARG;
  if (bytes > ((size_t)1 << 44)) return AKVQ_ERR_UNSUPPORTED;
  return hip_status(akvq::launch_stream_read(src, bytes, sink, non_temporal, static_cast<hipStream_t>(stream)));
}

size_t akvq_massive_workspace_bytes(int B, int T) {
  if (B <= 0 || T <= 0) return 0;
  return round_up((size_t)B * T * sizeof(float), 256);
}

int akvq_select_massive(const akvq_cache *c, const void *hidden, int T, int d_model, int top_k, float floor,
                        float *score_out, void *workspace, size_t workspace_bytes, void *stream) {
  int st = check_cache_shape(c);
  if (st != AKVQ_OK) return st;
  if (!c->sal_idx || !c->sal_cnt || !aligned16(c->sal_idx) || !aligned16(c->sal_cnt)) return AKVQ_ERR_INVALID_ARG;
  if (!hidden || !aligned16(hidden) || T <= 0 || T > c->T_cap || top_k <= 0 || d_model <= 0) return AKVQ_ERR_INVALID_ARG;
  if (d_model % 512 != 0) return AKVQ_ERR_UNSUPPORTED;
  if (top_k > c->S_cap) return AKVQ_ERR_CAPACITY;
  if (!(floor >= 0.0f)) return AKVQ_ERR_INVALID_ARG;
  if (score_out && !aligned16(score_out)) return AKVQ_ERR_INVALID_ARG;
  if (!score_out) {
    if (!workspace || !aligned16(workspace)) return AKVQ_ERR_INVALID_ARG;
    if (workspace_bytes < akvq_massive_workspace_bytes(c->B, T)) return AKVQ_ERR_WORKSPACE;
  }
  akvq::SelectArgs a{};
  a.sal_idx = c->sal_idx; a.sal_cnt = c->sal_cnt;
  a.B = c->B; a.Hkv = c->Hkv; a.Hq = c->Hkv; a.T = T; a.S_cap = c->S_cap; a.top_k = top_k;
  a.hidden = static_cast<const uint16_t *>(hidden);
  a.d_model = d_model; a.floor = floor; a.mass_per_batch = 1; a.skip_zero = 1;
  a.mass = score_out ? score_out : static_cast<float *>(workspace);
  return hip_status(akvq::launch_select_massive(a, static_cast<hipStream_t>(stream)));
}

static int check_window(const akvq_window *win) {
  if (!win) return AKVQ_OK;
  if (!win->k_win || !win->v_win || !aligned16(win->k_win) || !aligned16(win->v_win)) return AKVQ_ERR_INVALID_ARG;
  if (win->W <= 0 || win->W % 64 != 0) return AKVQ_ERR_INVALID_ARG;
  return AKVQ_OK;
}

static int check_rope(const akvq_rope *rope, uint32_t prerotated) {
  if (!rope) return AKVQ_OK;
  if (prerotated) return AKVQ_ERR_INVALID_ARG;  // the embedding precedes the rotation
  if (!rope->cos || !rope->sin || !aligned16(rope->cos) || !aligned16(rope->sin)) return AKVQ_ERR_INVALID_ARG;
  if (rope->batch_stride < 0 || rope->batch_stride % 8 != 0) return AKVQ_ERR_INVALID_ARG;
  return AKVQ_OK;
}

static int quantize_args(const akvq_cache *c, const void *k_new, const void *v_new, int n_src, int n_new,
                         float clip, float clip4, const int32_t *row_src, const uint8_t *row_tier,
                         uint32_t *fine_mask, const akvq_window *win, const akvq_rope *rope, uint32_t flags,
                         akvq::QuantArgs &a) {
  int st = check_rope(rope, flags & AKVQ_K_PREROTATED);
  if (st != AKVQ_OK) return st;
  st = check_cache_shape(c);
  if (st != AKVQ_OK) return st;
  st = check_cache_pointers(c);
  if (st != AKVQ_OK) return st;
  if (!k_new || !v_new || !aligned16(k_new) || !aligned16(v_new) || n_new <= 0 || n_src <= 0) return AKVQ_ERR_INVALID_ARG;
  if (!(clip > 0.0f) || clip > 1.0f || !(clip4 > 0.0f) || clip4 > 1.0f) return AKVQ_ERR_INVALID_ARG;
  if (too_many_units((long)c->B * c->Hkv)) return AKVQ_ERR_UNSUPPORTED;
  if ((long)c->T_len + n_new > c->T_cap) return AKVQ_ERR_CAPACITY;
  a = akvq::QuantArgs{};
  a.row_src = row_src; a.row_tier = row_tier; a.fine_mask = fine_mask; a.n_src = n_src; a.clip4 = clip4;
  st = check_window(win);
  if (st != AKVQ_OK) return st;
  if (win) { a.k_win = win->k_win; a.v_win = win->v_win; a.win_len = win->W; }
  if (rope) { a.rope_cos = rope->cos; a.rope_sin = rope->sin; a.rope_stride = rope->batch_stride; }
  a.k_new = static_cast<const uint16_t *>(k_new);
  a.v_new = static_cast<const uint16_t *>(v_new);
  a.k_codes = c->k_codes; a.v_codes = c->v_codes; a.k_meta = c->k_meta; a.v_meta = c->v_meta;
  a.k_sal = c->k_sal; a.v_sal = c->v_sal; a.sal_idx = c->sal_idx; a.sal_cnt = c->sal_cnt;
  a.Hkv = c->Hkv; a.T_cap = c->T_cap; a.S_cap = c->S_cap; a.T_len = c->T_len; a.n_new = n_new;
  a.first_blk = c->T_len / 32;
  a.n_blk = (c->T_len + n_new - 1) / 32 - a.first_blk + 1;
  a.clip = clip;
  a.rotate_k = (flags & AKVQ_K_PREROTATED) ? 0 : 1;
  a.rotate_v = (flags & AKVQ_V_PREROTATED) ? 0 : 1;
  return AKVQ_OK;
}

static int quantize_common(const akvq_cache *c, const void *k_new, const void *v_new, int n_src, int n_new,
                           float clip, float clip4, const int32_t *row_src, const uint8_t *row_tier,
                           uint32_t *fine_mask, const akvq_window *win, const akvq_rope *rope, uint32_t flags,
                           void *stream) {
  akvq::QuantArgs a;
  const int st = quantize_args(c, k_new, v_new, n_src, n_new, clip, clip4, row_src, row_tier, fine_mask, win, rope,
                               flags, a);
  if (st != AKVQ_OK) return st;
  return hip_status(akvq::launch_quantize_append(a, c->B, c->G, static_cast<hipStream_t>(stream)));
}

int akvq_quantize_append(const akvq_cache *c, const void *k_new, const void *v_new, int n_new, float clip,
                         uint32_t flags, void *stream) {
  return quantize_common(c, k_new, v_new, n_new, n_new, clip, 1.0f, nullptr, nullptr, nullptr, nullptr, nullptr, flags,
                         stream);
}

int akvq_quantize_append_tiered(const akvq_cache *c, const void *k_src, const void *v_src, int n_src,
                                const int32_t *row_src, const uint8_t *row_tier, int n_rows, float clip2,
                                float clip4, uint32_t *fine_mask, const akvq_window *win, uint32_t flags,
                                void *stream) {
  return akvq_quantize_append_rope(c, k_src, v_src, n_src, row_src, row_tier, n_rows, clip2, clip4, fine_mask, win,
                                   nullptr, flags, stream);
}

int akvq_quantize_append_rope(const akvq_cache *c, const void *k_src, const void *v_src, int n_src,
                              const int32_t *row_src, const uint8_t *row_tier, int n_rows, float clip2, float clip4,
                              uint32_t *fine_mask, const akvq_window *win, const akvq_rope *rope, uint32_t flags,
                              void *stream) {
  const bool mapped = row_src || row_tier || fine_mask;  // all three or none
  if (mapped && (!row_src || !row_tier || !fine_mask || !aligned16(row_src) || !aligned16(row_tier) ||
                 !aligned16(fine_mask)))
    return AKVQ_ERR_INVALID_ARG;
  if (!mapped && n_rows != n_src) return AKVQ_ERR_INVALID_ARG;
  return quantize_common(c, k_src, v_src, n_src, n_rows, clip2, clip4, row_src, row_tier, fine_mask, win, rope, flags,
                         stream);
}

int akvq_decode_attention(const akvq_cache *c, const void *q, int Hq, float sm_scale, void *out, float *lse_out,
                          int n_split, void *workspace, size_t workspace_bytes, uint32_t flags, void *stream) {
  return akvq_decode_attention_rope(c, nullptr, nullptr, q, nullptr, Hq, sm_scale, out, lse_out, n_split, workspace,
                                    workspace_bytes, flags, stream);
}

size_t akvq_decode_static_scratch_bytes(void) { return akvq::kDecodeStaticScratchBytes; }

int akvq_decode_attention_static(const akvq_cache *c, const void *q, int Hq, float sm_scale, void *out, float *lse_out,
                                 int n_split, uint32_t flags, void *stream) {
  // size check first, on the host, so that an oversize request launches nothing and touches no device state
  if (!c || c->B <= 0 || c->Hkv <= 0 || Hq <= 0) return AKVQ_ERR_INVALID_ARG;
  if (n_split <= 0) n_split = akvq_decode_default_splits(c->B, c->Hkv, c->T_len);
  if (n_split > 1024) return AKVQ_ERR_INVALID_ARG;
  if (akvq_decode_workspace_bytes(c->B, Hq, n_split) > akvq::kDecodeStaticScratchBytes) return AKVQ_ERR_WORKSPACE;
  void *ws = nullptr;
  const hipError_t e = akvq::decode_static_scratch(&ws);
  if (e != hipSuccess) return hip_status(e);
  return akvq_decode_attention_rope(c, nullptr, nullptr, q, nullptr, Hq, sm_scale, out, lse_out, n_split, ws,
                                    akvq::kDecodeStaticScratchBytes, flags, stream);
}

int akvq_decode_attention_tiered(const akvq_cache *c, const uint32_t *fine_mask, const akvq_window *win,
                                 const void *q, int Hq, float sm_scale, void *out, float *lse_out, int n_split,
                                 void *workspace, size_t workspace_bytes, uint32_t flags, void *stream) {
  return akvq_decode_attention_rope(c, fine_mask, win, q, nullptr, Hq, sm_scale, out, lse_out, n_split, workspace,
                                    workspace_bytes, flags, stream);
}

static int decode_args(const akvq_cache *c, const uint32_t *fine_mask, const akvq_window *win, const void *q,
                       const akvq_rope *rope, int Hq, float sm_scale, void *out, float *lse_out, int n_split,
                       void *workspace, size_t workspace_bytes, uint32_t flags, akvq::DecodeArgs &a) {
  if (fine_mask && !aligned16(fine_mask)) return AKVQ_ERR_INVALID_ARG;
  int st = check_rope(rope, flags & AKVQ_Q_PREROTATED);
  if (st != AKVQ_OK) return st;
  st = check_window(win);
  if (st != AKVQ_OK) return st;
  st = check_cache_shape(c);
  if (st != AKVQ_OK) return st;
  st = check_cache_pointers(c);
  if (st != AKVQ_OK) return st;
  if (c->T_len <= 0) return AKVQ_ERR_INVALID_ARG;
  if (!q || !out || !aligned16(q) || !aligned16(out)) return AKVQ_ERR_INVALID_ARG;
  if (lse_out && !aligned16(lse_out)) return AKVQ_ERR_INVALID_ARG;
  if (Hq <= 0 || Hq % c->Hkv != 0) return AKVQ_ERR_INVALID_ARG;
  if (Hq / c->Hkv > 8) return AKVQ_ERR_UNSUPPORTED;
  if (too_many_units((long)c->B * c->Hkv)) return AKVQ_ERR_UNSUPPORTED;
  if (n_split <= 0) n_split = akvq_decode_default_splits(c->B, c->Hkv, c->T_len);
  if (n_split > 1024) return AKVQ_ERR_INVALID_ARG;
  if (!workspace || !aligned16(workspace)) return AKVQ_ERR_INVALID_ARG;
  if (workspace_bytes < akvq_decode_workspace_bytes(c->B, Hq, n_split)) return AKVQ_ERR_WORKSPACE;
  a = akvq::DecodeArgs{};
  a.k_codes = c->k_codes; a.v_codes = c->v_codes; a.k_meta = c->k_meta; a.v_meta = c->v_meta;
  a.k_sal = c->k_sal; a.v_sal = c->v_sal; a.sal_idx = c->sal_idx; a.sal_cnt = c->sal_cnt;
  a.fine_mask = fine_mask;
  a.t_win = c->T_len;
  if (win) {
    a.k_win = win->k_win; a.v_win = win->v_win; a.win_len = win->W;
    a.t_win = (((c->T_len > win->W) ? c->T_len - win->W : 0) + 1) & ~1;  // even row at or above T_len - W
  }
  a.q = static_cast<const uint16_t *>(q);
  a.partial = static_cast<float *>(workspace);
  a.out = out; a.lse = lse_out;
  a.B = c->B; a.Hq = Hq; a.Hkv = c->Hkv; a.T_cap = c->T_cap; a.S_cap = c->S_cap; a.T_len = c->T_len;
  a.n_split = n_split; a.sm_scale = sm_scale;
  if (rope) { a.rope_cos = rope->cos; a.rope_sin = rope->sin; a.rope_stride = rope->batch_stride; }
  a.q_rotated = (flags & AKVQ_Q_PREROTATED) ? 1 : 0;
  a.out_rotated = (flags & AKVQ_OUT_ROTATED) ? 1 : 0;
  a.out_half = (flags & AKVQ_OUT_FP16) ? 1 : 0;
  return AKVQ_OK;
}

int akvq_decode_attention_rope(const akvq_cache *c, const uint32_t *fine_mask, const akvq_window *win, const void *q,
                               const akvq_rope *rope, int Hq, float sm_scale, void *out, float *lse_out, int n_split,
                               void *workspace, size_t workspace_bytes, uint32_t flags, void *stream) {
  akvq::DecodeArgs a;
  const int st = decode_args(c, fine_mask, win, q, rope, Hq, sm_scale, out, lse_out, n_split, workspace,
                             workspace_bytes, flags, a);
  if (st != AKVQ_OK) return st;
  return hip_status(akvq::launch_decode_attention(a, c->G, static_cast<hipStream_t>(stream)));
}

int akvq_decode_step(const akvq_cache *c, const uint32_t *fine_mask, const akvq_window *win, const void *k_new,
                     const void *v_new, const void *q, const akvq_rope *rope, int Hq, float clip, float sm_scale,
                     void *out, float *lse_out, int n_split, void *workspace, size_t workspace_bytes, uint32_t flags,
                     void *stream) {
  if (!c) return AKVQ_ERR_INVALID_ARG;
  akvq::QuantArgs qa;
  int st = quantize_args(c, k_new, v_new, 1, 1, clip, 1.0f, nullptr, nullptr, nullptr, win, rope, flags, qa);
  if (st != AKVQ_OK) return st;
  akvq_cache after = *c;  // what decode attends over: the cached rows and the new one
  after.T_len = c->T_len + 1;
  akvq::DecodeArgs a;
  st = decode_args(&after, fine_mask, win, q, rope, Hq, sm_scale, out, lse_out, n_split, workspace, workspace_bytes,
                   flags, a);
  if (st != AKVQ_OK) return st;
  a.fused_append = 1;
  a.step = qa;
  return hip_status(akvq::launch_decode_attention(a, c->G, static_cast<hipStream_t>(stream)));
}

}  // extern "C"

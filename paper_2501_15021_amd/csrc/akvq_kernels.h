// Host-side launch interfaces of the libakvq kernels (internal; the public ABI is include/akvq.h).
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

namespace akvq {

struct QuantArgs {
  const uint16_t *k_new, *v_new;  // [B][Hkv][n_new][128] binary16
  uint32_t *k_codes, *v_codes, *k_meta, *v_meta;
  uint16_t *k_sal, *v_sal;
  const int32_t *sal_idx, *sal_cnt;
  int Hkv, T_cap, S_cap, T_len, n_new;
  int first_blk, n_blk;  // 32-token blocks touched by rows [T_len, T_len + n_new)
  float clip;
  int rotate_k, rotate_v;
  // tiered append (all null / zero for the plain call): source row and tier of every new cache row, per batch element
  const int32_t *row_src;   // [B][n_new]
  const uint8_t *row_tier;  // [B][n_new]
  uint32_t *fine_mask;      // [B][T_cap/32]
  int n_src;                // rows per (b, kv-head) in k_new / v_new (= n_new for the plain call)
  float clip4;
  uint16_t *k_win, *v_win;  // recent-window rings (null: none)
  int win_len;
  const uint16_t *rope_cos, *rope_sin;  // rotary tables for pre-RoPE K rows (null: rows arrive embedded), [n_src][64] binary16
  long long rope_stride;                // elements between the tables of consecutive batch elements
  int skip_overlay;  // the block kernel leaves the 16-bit overlay rows to the overlay pass that follows it
};
hipError_t launch_quantize_append(const QuantArgs &a, int B, int G, hipStream_t stream);

struct DecodeArgs {
  const uint32_t *k_codes, *v_codes, *k_meta, *v_meta;
  const uint16_t *k_sal, *v_sal;
  const int32_t *sal_idx, *sal_cnt;
  const uint32_t *fine_mask;  // [B][T_cap/32] or null: fine halves of 4-bit tokens stored as row pairs
  const uint16_t *k_win, *v_win;  // recent-window rings (null: none), win_len slots
  int win_len;
  int t_win;                  // first row read from the rings (= T_len without a window)
  const uint16_t *q;  // [B][Hq][128] binary16
  float *partial;     // [B*Hq][n_split][kPartialStride] fp32
  void *out;          // [B][Hq][128] fp32, or binary16 when out_half
  float *lse;         // optional [B][Hq]
  int B, Hq, Hkv, T_cap, S_cap, T_len, n_split;
  float sm_scale;
  int q_rotated, out_rotated, out_half;
  // the decode step in one launch: row T_len - 1 is first quantized from step.k_new / step.v_new (step.T_len is that
  // row) by the workgroups of split append_split: the split whose tile range holds the tile of that row (see
  // decode_split_range), so that the row is written and read by the same workgroup.  They are also the only ones to
  // read 16-bit rows then.
  int fused_append;
  int append_split;
  QuantArgs step;
  const uint16_t *rope_cos, *rope_sin;  // rotary tables for pre-RoPE queries (null: none), one row of 64 per batch element
  long long rope_stride;
};
constexpr int kPartialStride = 132;  // m, l, 2 pad, 128 accumulators

// How the code stream's n_tiles tiles are dealt to the n_split KV splits: equal runs of ceil(n_tiles / n_split) tiles,
// so trailing splits can be short or empty.  Used by the kernels, by the host (append_split) and by the public helper
// akvq_decode_split_range, so that all three agree by construction.
__host__ __device__ inline int decode_tiles_per_split(int n_tiles, int n_split) {
  return n_tiles > 0 ? (n_tiles - 1) / n_split + 1 : 0;  // ceil(n_tiles / n_split) without overflow
}
__host__ __device__ inline void decode_split_range(int n_tiles, int n_split, int split, int &begin, int &end) {
  const int per = decode_tiles_per_split(n_tiles, n_split);
  const long long b = (long long)split * per, e = b + per;
  begin = (int)(b < n_tiles ? b : n_tiles);
  end = (int)(e < n_tiles ? e : n_tiles);
}
// the split whose range holds the last tile (the tile of the row a fused decode step appends); split 0 if there is no tile
__host__ __device__ inline int decode_last_tile_split(int n_tiles, int n_split) {
  if (n_tiles <= 0) return 0;
  return (n_tiles - 1) / decode_tiles_per_split(n_tiles, n_split);
}
constexpr int kMhaTileRows = 64, kGqaTileRows = 32;  // rows per code-stream tile of the two decode kernels
hipError_t launch_decode_attention(const DecodeArgs &a, int G, hipStream_t stream);
// Device address, on the current device, of the library's fixed scratch array for split-KV partials (no allocation).
constexpr size_t kDecodeStaticScratchBytes = 8u << 20;
hipError_t decode_static_scratch(void **ptr);

struct SelectArgs {
  const uint8_t *is_text;    // [B][T]
  const uint16_t *q_tail;    // [B][Hq][W][128] binary16
  const uint16_t *k;         // [B][Hkv][T][128] binary16
  int32_t *sal_idx, *sal_cnt;
  float *mass;               // [B][Hkv][T] fp32 (user buffer or workspace)
  float *row_stats;          // workspace: [B][Hq][n_chunk][W][2]
  int B, Hq, Hkv, T, W, top_k, S_cap, n_chunk;
  float sm_scale;
  // massive-activation mode: hidden states, one score row per batch element, zero keys are never selected
  const uint16_t *hidden;    // [B][T][d_model] binary16
  int d_model;
  float floor;
  int mass_per_batch;        // top-k reads mass[b][T] (shared by the batch element's kv-heads) instead of mass[b][hkv][T]
  int skip_zero;
  float *mass_shared;        // token-level pivots: [B][T] sums of the kv-heads' masses (workspace), null: per-head lists
};
constexpr int kScoreChunk = 2048;  // keys per scoring workgroup
hipError_t launch_select_tsa(const SelectArgs &a, hipStream_t stream);
hipError_t launch_select_psa(const SelectArgs &a, hipStream_t stream);
hipError_t launch_select_massive(const SelectArgs &a, hipStream_t stream);

// offline fold of H_128 into a projection matrix w [rows][cols] binary16 (axis 1: runs of 128 columns, axis 0: of rows)
hipError_t launch_fold_hadamard(const uint16_t *w, uint16_t *out, int rows, int cols, int axis, hipStream_t stream);

// measurement aid: plain 128-bit streaming read of `bytes` bytes (a multiple of 16, at least 16)
hipError_t launch_stream_read(const void *src, size_t bytes, uint32_t *sink, int non_temporal, hipStream_t stream);

}  // namespace akvq

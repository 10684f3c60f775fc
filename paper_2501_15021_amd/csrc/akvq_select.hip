// Salient-token identification (Section III-B of arXiv 2501.15021).
//   TSA layers: the salient set is the text positions -> ordered stream compaction of the modality mask.
//   PSA layers: pivot tokens are the few tokens that receive most of the attention (Section I / III-A.3); the score
//   is the attention-column mass of the last W prompt rows, computed on the matrix cores (bfloat16 operands, fp32
//   accumulate, fp32 softmax) in two streaming passes over K (row statistics, then column sums), followed by an
//   exact top-k (radix select on the fp32 bit patterns, ties to the lower position).
#include <atomic>

#include "akvq_device.h"
#include "akvq_kernels.h"

namespace akvq {

namespace {

// ---- ordered compaction helpers (256-thread workgroup) -----------------------------------------------
// exclusive prefix of a 0/1 flag over the workgroup, plus the workgroup total
__device__ __forceinline__ int block_flag_scan(bool flag, int *wave_tot, int &total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const unsigned long long ballot = __ballot(flag);
  const int within = __popcll(ballot & ((1ull << lane) - 1ull));
  __syncthreads();  // previous use of wave_tot finished
  if (lane == 0) wave_tot[wave] = __popcll(ballot);
  __syncthreads();
  int before = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < 4; ++w) {
    const int c = wave_tot[w];
    if (w < wave) before += c;
    tot += c;
  }
  total = tot;
  return before + within;
}

__global__ __launch_bounds__(256) void select_tsa_kernel(SelectArgs a) {
  __shared__ int wave_tot[4];
  const int bh = blockIdx.x, b = bh / a.Hkv;
  const uint8_t *mask = a.is_text + (size_t)b * a.T;
  int32_t *out = a.sal_idx + (size_t)bh * a.S_cap;
  int base_count = 0;
  for (int base = 0; base < a.T; base += 256) {
    const int t = base + threadIdx.x;
    const bool flag = t < a.T && mask[t] != 0;
    int total;
    const int pos = base_count + block_flag_scan(flag, wave_tot, total);
    if (flag && pos < a.S_cap) out[pos] = t;
    base_count += total;
  }
  if (threadIdx.x == 0) a.sal_cnt[bh] = base_count;
}

// ---- pivot scoring ---------------------------------------------------------------------------------------
// Scoring windows of fewer than 64 rows (the kernels for W = 64 follow further down): each workgroup (4 wavefronts)
// owns kScoreChunk consecutive keys of one (batch, query head); its wavefronts take the groups of 16 keys in turn,
// with the next groups' loads in flight while the current one goes through the matrix cores.
// Logits are kept in the base-2 domain (sm_scale * log2(e) folded into one multiply) so that exponentials are bare
// v_exp_f32; both passes use the same domain, so the statistics carry over unchanged.
constexpr int kGroupsPerWave = kScoreChunk / (4 * 16);
constexpr int kKeyDepth = 1;  // key groups in flight ahead of the one being scored in the second pass (deeper is slower)
static_assert(kGroupsPerWave % (kKeyDepth + 1) == 0, "the scoring loop is unrolled over the key ring");

// binary16 pair (packed) -> bfloat16 pair (packed), each rounded to nearest even
__device__ __forceinline__ uint32_t half2_to_bf16x2(uint32_t hh) {
  return pack_bf16x2(half_bits_to_float(hh & 0xFFFFu), half_bits_to_float(hh >> 16));
}
__device__ __forceinline__ bf16x8 rows8_as_bf16(u32x4 raw) {
  u32x4 r = {half2_to_bf16x2(raw[0]), half2_to_bf16x2(raw[1]), half2_to_bf16x2(raw[2]), half2_to_bf16x2(raw[3])};
  return __builtin_bit_cast(bf16x8, r);
}

struct KeyGroup {
  u32x4 raw[4];  // 16 keys x 128 channels as this lane's four 8-channel pieces (binary16)
};
__device__ __forceinline__ void load_key_group(const uint16_t *k_rows, int t_first, int T, int mrow, int qd, KeyGroup &g) {
  const int t = min(t_first + mrow, T - 1);  // rows past the end repeat the last key; the causal mask removes them
#pragma unroll
  for (int kc = 0; kc < 4; ++kc)
    g.raw[kc] = *reinterpret_cast<const u32x4 *>(k_rows + (size_t)t * kD + 32 * kc + 8 * qd);
}

// The same 16 keys as they come from memory line by line: load i covers keys 4i .. 4i+3 whole, lane l taking the
// (l % 16)-th 16-byte piece of key 4i + l / 16, so every load is 1 KB of consecutive bytes (eight full cache lines, each
// fetched by one instruction only) and can carry the non-temporal hint.
__device__ __forceinline__ void load_key_lines(const uint16_t *k_rows, int t_first, int T, int lane, KeyGroup &g) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int t = min(t_first + 4 * i + (lane >> 4), T - 1);  // rows past the end repeat the last key; the causal mask removes them
    g.raw[i] = stream_load(reinterpret_cast<const u32x4 *>(k_rows + (size_t)t * kD + 8 * (lane & 15)));
  }
}
// ... turned into matrix-core operands through the wavefront's own 4 KB of LDS (converted to bfloat16 on the way in):
// piece p of key r sits at slot r * 16 + (p ^ r), which keeps both the writes (16 pieces of one key) and the reads (one
// piece of 16 keys) free of bank conflicts.  Same wavefront on both sides; its LDS instructions complete in order.
__device__ __forceinline__ void lines_to_operands(const KeyGroup &g, u32x4 *tile, int lane, bf16x8 (&kb)[4]) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int r = 4 * i + (lane >> 4), p = lane & 15;
    tile[r * 16 + (p ^ r)] = __builtin_bit_cast(u32x4, rows8_as_bf16(g.raw[i]));
  }
  const int mrow = lane & 15, qd = lane >> 4;
#pragma unroll
  for (int kc = 0; kc < 4; ++kc) kb[kc] = __builtin_bit_cast(bf16x8, tile[mrow * 16 + ((4 * kc + qd) ^ mrow)]);
}
// products of such operands with the query rows in LDS, keys as the first operand: acc[rb][i] = key 4*qd + i of the
// group, tail row 16*rb + mrow (the query operands are re-read per group behind an opaque offset, see score_16keys)
template <int NRB>
__device__ __forceinline__ void score_operands_by_row(const u32x4 *q_lds, const bf16x8 (&kb)[4], int mrow, int qd,
                                                      f32x4 (&acc)[4]) {
  uint32_t lane_off = (uint32_t)(qd * 16 + mrow);
  asm volatile("" : "+v"(lane_off));
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) {
    acc[rb] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kc = 0; kc < 4; ++kc)
      acc[rb] = mfma_bf16(kb[kc], __builtin_bit_cast(bf16x8, q_lds[(rb * 4 + kc) * 64 + lane_off]), acc[rb]);
  }
}
// dot products of the W tail rows of one query head with 16 keys: acc[rb][i] = row 16*rb + 4*qd + i, key = mrow
template <int NRB>
__device__ __forceinline__ void score_16keys(const u32x4 *q_lds, const KeyGroup &g, int mrow, int qd, f32x4 (&acc)[4]) {
  // The query operands live in LDS and are re-read for every key group: the offset is made opaque so the reads are
  // not hoisted out of the caller's loop into 64 registers (which would cost a wavefront of occupancy).
  uint32_t lane_off = (uint32_t)(qd * 16 + mrow);
  asm volatile("" : "+v"(lane_off));
  bf16x8 kb[4];
#pragma unroll
  for (int kc = 0; kc < 4; ++kc) kb[kc] = rows8_as_bf16(g.raw[kc]);
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) {
    acc[rb] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kc = 0; kc < 4; ++kc)
      acc[rb] = mfma_bf16(__builtin_bit_cast(bf16x8, q_lds[(rb * 4 + kc) * 64 + lane_off]), kb[kc], acc[rb]);
  }
}
// causal visibility of key t for tail row `row` (the row sits at position T-W+row); keys past the end are never seen
__device__ __forceinline__ bool key_seen(int t, int row, int T, int W) { return t < T && t <= T - W + row; }
// a group of 16 keys starting at t_first needs per-element masking only if it reaches past position T-W
__device__ __forceinline__ bool group_has_masked(int t_first, int T, int W) { return t_first + 15 > T - W; }

// the W tail rows of one query head as matrix-core A operands in LDS: slot (rb, kc, lane) is what lane (mrow, qd)
// feeds for row block rb and channel step kc; wavefront w converts row blocks w, w+4, ...
template <int NRB>
__device__ __forceinline__ void stage_query_rows(const uint16_t *q_head, int wave, int mrow, int qd, u32x4 *q_lds) {
  for (int rb = wave; rb < NRB; rb += 4)
#pragma unroll
    for (int kc = 0; kc < 4; ++kc)
      q_lds[(rb * 4 + kc) * 64 + qd * 16 + mrow] = __builtin_bit_cast(u32x4, rows8_as_bf16(
          *reinterpret_cast<const u32x4 *>(q_head + (size_t)(16 * rb + mrow) * kD + 32 * kc + 8 * qd)));
}

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLazyRaise = 12.0f;  // a row reference is raised only for logits this far (base 2) above it
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }  // bare v_exp_f32

// ---- row statistics of the first pass, key-major ---------------------------------------------------------------
// The products are taken with the keys as the first operand: acc[rb][i] = key 4*qd + i of the group against tail row
// row0 + 16*rb + mrow, so a lane holds four keys of ONE tail row per row block, and a row's reference m and partial sum l
// are one register each (shared with the three other lanes of the row) instead of four.
// m is a reference, not the running maximum: it is raised only when a logit exceeds it by more than kLazyRaise (or at
// the causal edge), so in the common case the sums just grow; otherwise the references are raised to the row maxima
// of the group and the sums rescaled.
struct RowStats {
  float m[4], l[4];
};
template <int NRB>
__device__ __forceinline__ void stats_raise_and_add(RowStats &s, const f32x4 (&acc)[4], float scale2, int t_first, int T,
                                                    int W, int mrow, int qd, int row0 = 0) {
  int t = t_first + 4 * qd;
  asm volatile("" : "+v"(t));  // keeps the masks from being precomputed ahead of the loop
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) {
    float sv[4];
    bool seen[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      seen[i] = key_seen(t + i, row0 + 16 * rb + mrow, T, W);
      sv[i] = seen[i] ? scale2 * acc[rb][i] : -INFINITY;
    }
    float top = fmaxf(fmaxf(sv[0], sv[1]), fmaxf(sv[2], sv[3]));
    top = fmaxf(top, __shfl_xor(top, 16, kWave));
    top = fmaxf(top, __shfl_xor(top, 32, kWave));
    if (top > s.m[rb]) {  // uniform over the row's four lanes; a reference of -inf goes with a zero sum
      s.l[rb] *= fast_exp2(s.m[rb] - top);
      s.m[rb] = top;
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
      if (seen[i]) s.l[rb] += fast_exp2(sv[i] - s.m[rb]);
  }
}
// a group every key of which is seen by every tail row
template <int NRB>
__device__ __forceinline__ void stats_add_group(RowStats &s, const f32x4 (&acc)[4], float scale2, int t_first, int T,
                                                int W, int mrow, int qd, int row0 = 0) {
  float x[4][4];
  float top = -INFINITY;
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      x[rb][i] = __builtin_fmaf(acc[rb][i], scale2, -s.m[rb]);
      top = fmaxf(top, x[rb][i]);
    }
  if (__ballot(!(top <= kLazyRaise)) == 0ull) {
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
      s.l[rb] += (fast_exp2(x[rb][0]) + fast_exp2(x[rb][1])) + (fast_exp2(x[rb][2]) + fast_exp2(x[rb][3]));
  } else {
    stats_raise_and_add<NRB>(s, acc, scale2, t_first, T, W, mrow, qd, row0);
  }
}
// the row's four lanes share the reference: their sums add up (lanes of quarter 0 hold the result)
__device__ __forceinline__ float stats_row_sum(float l) {
  l += __shfl_xor(l, 16, kWave);
  l += __shfl_xor(l, 32, kWave);
  return l;
}

// pass 1: per (b, hq, chunk): reference and sum of exponentials (base 2) of every tail row
constexpr int kStatsDepth = 3;  // key groups in flight ahead of the one being scored in the first pass
static_assert(kGroupsPerWave % (kStatsDepth + 1) == 0, "the scoring loop is unrolled over the key ring");
template <int NRB>
__global__ __launch_bounds__(256, 4) void psa_row_stats_kernel(SelectArgs a) {  // 4 wavefronts per SIMD: at most 128 registers
  __shared__ float st_m[4][64], st_l[4][64];
  const int chunk = blockIdx.x, bhq = blockIdx.y;
  const int b = bhq / a.Hq, hq = bhq % a.Hq, hkv = hq / (a.Hq / a.Hkv);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, mrow = lane & 15, qd = lane >> 4;
  const uint16_t *k_rows = a.k + ((size_t)b * a.Hkv + hkv) * a.T * kD;
  const float scale2 = a.sm_scale * kLog2e;
  __shared__ u32x4 q_lds[NRB * 4 * 64];
  __shared__ u32x4 key_tile[4][256];
  // the wavefronts take the chunk's groups of 16 keys in turn, so the workgroup walks its keys front to back in 16 KB
  // windows (a quarter of the chunk per wavefront, i.e. four distant streams per workgroup, is 3-4 % slower on HBM)
  const int t_wave = chunk * kScoreChunk + wave * 16;
  // kStatsDepth groups of keys are in flight ahead of the one being scored (a ring of register buffers; loads are
  // unconditional with clamped addresses, so the wait counts the compiler derives stay exact).  The first keys are
  // requested before the query rows are staged, so the two latencies overlap.  The keys come line by line with the
  // non-temporal hint and are turned into operands through LDS (2-4 % of the pass; the second pass would lose a
  // workgroup per CU to the extra 16 KB and keeps its direct half-line loads).
  KeyGroup ring[kStatsDepth + 1];
#pragma unroll
  for (int p = 0; p < kStatsDepth; ++p) load_key_lines(k_rows, t_wave + 64 * p, a.T, lane, ring[p]);
  stage_query_rows<NRB>(a.q_tail + (size_t)bhq * a.W * kD, wave, mrow, qd, q_lds);
  __syncthreads();
  RowStats st;  // of tail row 16*rb + mrow, over the keys 4*qd .. 4*qd + 3 of every group
#pragma unroll
  for (int rb = 0; rb < 4; ++rb) { st.m[rb] = -INFINITY; st.l[rb] = 0.0f; }
  for (int g0 = 0; g0 < kGroupsPerWave; g0 += kStatsDepth + 1)
#pragma unroll
  for (int u = 0; u <= kStatsDepth; ++u) {
    const int g = g0 + u;
    const int t_first = t_wave + 64 * g;
    load_key_lines(k_rows, t_wave + 64 * min(g + kStatsDepth, kGroupsPerWave - 1), a.T, lane,
                   ring[(u + kStatsDepth) % (kStatsDepth + 1)]);
    if (t_first >= a.T) continue;  // uniform over the wavefront
    f32x4 acc[4];
    bf16x8 kb[4];
    lines_to_operands(ring[u], key_tile[wave], lane, kb);
    score_operands_by_row<NRB>(q_lds, kb, mrow, qd, acc);
    if (!group_has_masked(t_first, a.T, a.W)) stats_add_group<NRB>(st, acc, scale2, t_first, a.T, a.W, mrow, qd);
    else stats_raise_and_add<NRB>(st, acc, scale2, t_first, a.T, a.W, mrow, qd);
  }
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) {
    const float lr = stats_row_sum(st.l[rb]);
    if (qd == 0) { st_m[wave][16 * rb + mrow] = st.m[rb]; st_l[wave][16 * rb + mrow] = lr; }
  }
  __syncthreads();
  if (threadIdx.x < a.W) {
    const int row = threadIdx.x;
    float mm = -INFINITY;
#pragma unroll
    for (int w = 0; w < 4; ++w) mm = fmaxf(mm, st_m[w][row]);
    float ll = 0.0f;
#pragma unroll
    for (int w = 0; w < 4; ++w)
      if (st_m[w][row] != -INFINITY) ll += st_l[w][row] * fast_exp2(st_m[w][row] - mm);
    float *dst = a.row_stats + (((size_t)bhq * a.n_chunk + chunk) * a.W + row) * 2;
    dst[0] = mm;
    dst[1] = ll;
  }
}

// pass 2: per (b, hkv, chunk): mass[t] = sum over the group's heads and the tail rows of 2^(s - m_row) / l_row
template <int NRB>
__global__ __launch_bounds__(256, 4) void psa_mass_kernel(SelectArgs a) {  // registers and LDS sized for 4 workgroups per CU
  __shared__ __attribute__((aligned(16))) float row_m[64], row_il[64];
  __shared__ u32x4 q_lds[NRB * 4 * 64];
  const int chunk = blockIdx.x, bh = blockIdx.y;
  const int b = bh / a.Hkv, hkv = bh % a.Hkv, R = a.Hq / a.Hkv;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, mrow = lane & 15, qd = lane >> 4;
  const uint16_t *k_rows = a.k + (size_t)bh * a.T * kD;
  const float scale2 = a.sm_scale * kLog2e;
  const int t_wave = chunk * kScoreChunk + wave * 16;  // groups of 16 keys dealt to the wavefronts in turn
  // column sums of the chunk, one slot per (pair of row quarters, key): the two quarters of a pair are added across
  // lanes first, every slot then has a single owning lane, so the sums over key groups and over the heads of the
  // group are plain read-add-write in a fixed order
  __shared__ float col_lds[2 * kScoreChunk];
  for (int i = threadIdx.x; i < 2 * kScoreChunk; i += 256) col_lds[i] = 0.0f;
  for (int h = 0; h < R; ++h) {
    const int bhq = b * a.Hq + hkv * R + h;
    KeyGroup ring[kKeyDepth + 1];  // first keys requested before the row statistics and query rows are staged
#pragma unroll
    for (int p = 0; p < kKeyDepth; ++p) load_key_group(k_rows, t_wave + 64 * p, a.T, mrow, qd, ring[p]);
    __syncthreads();
    if (threadIdx.x < a.W) {  // merge the chunk statistics of this row
      const int row = threadIdx.x;
      const float *src = a.row_stats + ((size_t)bhq * a.n_chunk * a.W + row) * 2;
      float mm = -INFINITY;
      for (int c = 0; c < a.n_chunk; ++c) mm = fmaxf(mm, src[(size_t)c * a.W * 2]);
      float ll = 0.0f;
      for (int c = 0; c < a.n_chunk; ++c) {
        const float mc = src[(size_t)c * a.W * 2];
        if (mc != -INFINITY) ll += src[(size_t)c * a.W * 2 + 1] * fast_exp2(mc - mm);
      }
      row_m[row] = mm;
      row_il[row] = 1.0f / ll;
    }
    stage_query_rows<NRB>(a.q_tail + (size_t)bhq * a.W * kD, wave, mrow, qd, q_lds);
    __syncthreads();
#pragma unroll
    for (int p = 0; p < kKeyDepth; ++p)
#pragma unroll
      for (int kc = 0; kc < 4; ++kc) settle(ring[p].raw[kc]);
    for (int g0 = 0; g0 < kGroupsPerWave; g0 += kKeyDepth + 1)
#pragma unroll
    for (int u = 0; u <= kKeyDepth; ++u) {
      const int g = g0 + u;
      const int t_first = t_wave + 64 * g;
      load_key_group(k_rows, t_wave + 64 * min(g + kKeyDepth, kGroupsPerWave - 1), a.T, mrow, qd,
                     ring[(u + kKeyDepth) % (kKeyDepth + 1)]);
      if (t_first >= a.T) continue;  // uniform over the wavefront
      const KeyGroup &cur = ring[u];
      f32x4 acc[4];
      score_16keys<NRB>(q_lds, cur, mrow, qd, acc);
      uint32_t row_off = (uint32_t)(4 * qd);  // opaque for the same reason as the query operands
      asm volatile("" : "+v"(row_off));
      const bool masked = group_has_masked(t_first, a.T, a.W);  // uniform over the wavefront
      float c0 = 0.0f, c1 = 0.0f;  // two chains: even and odd row blocks
#pragma unroll
      for (int rb = 0; rb < NRB; ++rb) {
        const f32x4 rm = *reinterpret_cast<const f32x4 *>(row_m + 16 * rb + row_off);
        const f32x4 ril = *reinterpret_cast<const f32x4 *>(row_il + 16 * rb + row_off);
        float &c = (rb & 1) ? c1 : c0;
        if (!masked) {
#pragma unroll
          for (int i = 0; i < 4; ++i)
            c = __builtin_fmaf(fast_exp2(__builtin_fmaf(acc[rb][i], scale2, -rm[i])), ril[i], c);
        } else {
          int t = t_first + mrow;
          asm volatile("" : "+v"(t));  // keeps the masks of all groups from being precomputed ahead of the loop
#pragma unroll
          for (int i = 0; i < 4; ++i)
            if (key_seen(t, 16 * rb + 4 * qd + i, a.T, a.W))
              c = __builtin_fmaf(fast_exp2(__builtin_fmaf(acc[rb][i], scale2, -rm[i])), ril[i], c);
        }
      }
      float c = c0 + c1;
      c += __shfl_xor(c, 16, kWave);  // quarters qd and qd ^ 1
      if ((qd & 1) == 0) {
        float *slot = col_lds + (qd >> 1) * kScoreChunk + (t_first - chunk * kScoreChunk) + mrow;
        *slot += c;
      }
    }
  }
  __syncthreads();
  for (int i = threadIdx.x; i < kScoreChunk; i += 256) {
    const int t = chunk * kScoreChunk + i;
    if (t < a.T)
      a.mass[(size_t)bh * a.T + t] = col_lds[i] + col_lds[kScoreChunk + i];
  }
}

// ---- pivot scoring, W = 64: scoring wavefronts with their rows in registers, keys fed through LDS -----------------
// (any number of query heads per KV head up to eight; the kernels above serve the other W)
// One workgroup per (batch, kv-head, chunk of kScoreChunk keys) with one or two wavefronts per query head of the group,
// each holding all or half of the head's W = 64 tail rows in registers as one matrix operand.  The keys are read from
// HBM and converted to bfloat16 once for the whole group: blocks of 64 keys go through LDS (two buffers, laid out as
// matrix-core operands) and every scoring wavefront multiplies all of them with its rows.  Per block: the keys of the
// block after next are requested into registers, the next block's are converted and stored to LDS, the current block
// is scored; one barrier per block orders the buffers.  With fewer than eight heads per KV head the keys are brought
// in by wavefronts of their own (feeders: two in the first pass, one in the second, which also adds up the column
// sums); with eight heads the scoring wavefronts share that work.
// The first pass runs two wavefronts per head (32 rows and under 128 registers each, four wavefronts per SIMD: 10 %
// faster than one per head at about 200 registers and two per SIMD); the second pass one per head (with two, every
// key operand is read from LDS twice for half the arithmetic each time: 17 % slower), except with a single head.
// The feeders read whole keys (1 KB of consecutive bytes per load, non-temporal); against the kernels above, whose
// wavefronts load, convert and score their own keys, that is 2-7 % per pass with one head per KV head.
constexpr int kGqaBlockGroups = 4;                                // groups of 16 keys per block
constexpr int kGqaBlockKeys = 16 * kGqaBlockGroups;               // 64
constexpr int kGqaBlocks = kScoreChunk / kGqaBlockKeys;           // blocks per chunk
constexpr int kGqaItems = kGqaBlockGroups * 4;                    // 1 KB pieces (four whole keys each) of a block
constexpr int kGqaMaxHeads = 8;                                   // query heads per KV head
constexpr int kGqaFeederItems = kGqaItems / 2;                    // MAXIT from this on: feeder wavefronts bring in the keys
static_assert(kScoreChunk % kGqaBlockKeys == 0, "a chunk is a whole number of blocks");
static_assert(kGqaBlockGroups % 2 == 0, "the first pass walks a block two groups at a time");
static_assert(kGqaItems % (2 * kGqaMaxHeads) == 0, "up to sixteen scoring wavefronts share a block's pieces evenly");

// MAXIT: pieces of a block one wavefront brings in: pieces first, first + stride, ... (all of them for the feeder;
// kGqaItems / (scoring wavefronts) each when eight heads' scoring wavefronts share the work).  The loads are unconditional and in
// straight-line code, so that they are in flight together (under per-piece branches the wait counts the compiler
// inserts serialise them).
template <int MAXIT>
struct KeyStage {
  u32x4 raw[MAXIT];
};
template <int MAXIT>
__device__ __forceinline__ void request_block(const uint16_t *k_rows, int t_block, int T, int first, int stride, int mrow,
                                              int qd, KeyStage<MAXIT> &st) {
  // piece `item` of a block = keys 4*item .. 4*item + 3 whole: lane l takes the (l % 16)-th 16 bytes of key
  // 4*item + l / 16, so a load is 1 KB of consecutive bytes and can carry the non-temporal hint (every key is read
  // once per pass)
  const int lane = qd * 16 + mrow;
#pragma unroll
  for (int it = 0; it < MAXIT; ++it) {
    const int item = first + it * stride;  // uniform over the wavefront
    const int t = min(t_block + 4 * item + (lane >> 4), T - 1);  // rows past the end repeat the last key; never scored unmasked
    st.raw[it] = stream_load(reinterpret_cast<const u32x4 *>(k_rows + (size_t)t * kD + 8 * (lane & 15)));
  }
}
template <int MAXIT>
__device__ __forceinline__ void deposit_block(const KeyStage<MAXIT> &st, u32x4 *buf, int first, int stride, int lane) {
  // LDS layout of a block: key r of the block at r * 16 slots of 16 bytes, its piece p at slot p ^ (r % 16): the
  // writes here (16 pieces of one key per 16 lanes) and the operand reads (one piece of 16 keys) are both free of
  // bank conflicts
#pragma unroll
  for (int it = 0; it < MAXIT; ++it) {
    const int r = 4 * (first + it * stride) + (lane >> 4), p = lane & 15;
    buf[r * 16 + (p ^ (r & 15))] = __builtin_bit_cast(u32x4, rows8_as_bf16(st.raw[it]));
  }
}
// NRB row blocks of one query head, from row block rb0 on, as matrix-core operands in registers: q[rb * 4 + kc] is
// what this lane feeds for row block rb0 + rb and channel step kc
template <int NRB>
__device__ __forceinline__ void load_query_rows(const uint16_t *q_head, int rb0, int mrow, int qd, bf16x8 (&q)[NRB * 4]) {
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
    for (int kc = 0; kc < 4; ++kc)
      q[rb * 4 + kc] = rows8_as_bf16(
          *reinterpret_cast<const u32x4 *>(q_head + (size_t)(16 * (rb0 + rb) + mrow) * kD + 32 * kc + 8 * qd));
}
// One group of 16 keys of a block against the wavefront's rows: the keys' operands are read from LDS
// (read_block_group) and multiplied (products_of_group) in two steps, so that loops can read a group ahead of its
// products.  Row-major: acc[rb][i] = row 16*rb + 4*qd + i of the wavefront's rows, key mrow; BY_ROW swaps the
// operands: acc[rb][i] = key 4*qd + i of the group, row 16*rb + mrow.
__device__ __forceinline__ void read_block_group(const u32x4 *buf, int g, int lane, bf16x8 (&kb)[4]) {
  const int mrow = lane & 15, qd = lane >> 4;  // key 16*g + mrow of the block, channel pieces 4*kc + qd
#pragma unroll
  for (int kc = 0; kc < 4; ++kc) kb[kc] = __builtin_bit_cast(bf16x8, buf[(16 * g + mrow) * 16 + ((4 * kc + qd) ^ mrow)]);
}
template <int NRB, bool BY_ROW>
__device__ __forceinline__ void products_of_group(const bf16x8 (&q)[NRB * 4], const bf16x8 (&kb)[4], f32x4 (&acc)[4]) {
  // channel step outermost: consecutive products belong to different row blocks, so none waits for the one before it
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) acc[rb] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
  for (int kc = 0; kc < 4; ++kc)
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
      acc[rb] = BY_ROW ? mfma_bf16(kb[kc], q[rb * 4 + kc], acc[rb]) : mfma_bf16(q[rb * 4 + kc], kb[kc], acc[rb]);
}
template <int NRB, bool BY_ROW>
__device__ __forceinline__ void score_block_group(const bf16x8 (&q)[NRB * 4], const u32x4 *buf, int g, int lane,
                                                  f32x4 (&acc)[4]) {
  bf16x8 kb[4];
  read_block_group(buf, g, lane, kb);
  products_of_group<NRB, BY_ROW>(q, kb, acc);
}

// pass 1: per (b, hq, chunk): reference and sum of exponentials (base 2) of every tail row, as psa_row_stats_kernel.
// NRB: row blocks per wavefront (4: one wavefront per head; 2: two).
template <int NRB, int MAXIT>
__global__ __launch_bounds__(64 * kGqaMaxHeads * (4 / NRB)) void psa_row_stats_gqa_kernel(SelectArgs a) {
  constexpr int kHeadWaves = 4 / NRB;                      // wavefronts per query head
  constexpr int kMaxWaves = kGqaMaxHeads * kHeadWaves;     // scoring wavefronts of a workgroup, at most
  __shared__ u32x4 kbuf[2][kGqaItems * 64];
  const int chunk = blockIdx.x, bh = blockIdx.y;
  const int R = a.Hq / a.Hkv, b = bh / a.Hkv, hkv = bh % a.Hkv;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, mrow = lane & 15, qd = lane >> 4;
  const int n_score = R * kHeadWaves;                 // scoring wavefronts
  const int head = wave / kHeadWaves, rb0 = (wave % kHeadWaves) * NRB;  // this wavefront's head and first row block
  const int bhq = b * a.Hq + hkv * R + head;
  const uint16_t *k_rows = a.k + (size_t)bh * a.T * kD;
  const float scale2 = a.sm_scale * kLog2e;
  const int t_chunk = chunk * kScoreChunk;
  const int n_blk = min(kGqaBlocks, (a.T - t_chunk + kGqaBlockKeys - 1) / kGqaBlockKeys);  // blocks that hold keys
  // feeders (kGqaItems / MAXIT wavefronts behind the scoring ones) take consecutive pieces; without feeders the
  // scoring wavefronts take pieces wave, wave + kMaxWaves, ...
  constexpr bool kFeeder = MAXIT >= kGqaFeederItems;
  const int first = kFeeder ? (wave - n_score) * MAXIT : wave, stride = kFeeder ? 1 : kMaxWaves;
  KeyStage<MAXIT> st;
  if (kFeeder && wave >= n_score) {  // a feeder: same barriers as the scoring wavefronts below
    request_block(k_rows, t_chunk, a.T, first, stride, mrow, qd, st);
    deposit_block(st, kbuf[0], first, stride, lane);
    request_block(k_rows, t_chunk + kGqaBlockKeys, a.T, first, stride, mrow, qd, st);
    __syncthreads();
    for (int j = 0; j < n_blk; ++j) {
      if (j + 1 < n_blk) deposit_block(st, kbuf[(j + 1) & 1], first, stride, lane);
      if (j + 2 < n_blk) request_block(k_rows, t_chunk + (j + 2) * kGqaBlockKeys, a.T, first, stride, mrow, qd, st);
      __syncthreads();
    }
    return;
  }
  if constexpr (!kFeeder) request_block(k_rows, t_chunk, a.T, first, stride, mrow, qd, st);
  bf16x8 q[NRB * 4];
  load_query_rows<NRB>(a.q_tail + (size_t)bhq * a.W * kD, rb0, mrow, qd, q);
  if constexpr (!kFeeder) {
    deposit_block(st, kbuf[0], first, stride, lane);
    request_block(k_rows, t_chunk + kGqaBlockKeys, a.T, first, stride, mrow, qd, st);
  }
  RowStats st_row;  // of tail row 16*(rb0 + rb) + mrow, over the keys 4*qd .. 4*qd + 3 of every group
#pragma unroll
  for (int rb = 0; rb < 4; ++rb) { st_row.m[rb] = -INFINITY; st_row.l[rb] = 0.0f; }
  __syncthreads();
  for (int j = 0; j < n_blk; ++j) {
    if constexpr (!kFeeder) {
      if (j + 1 < n_blk) deposit_block(st, kbuf[(j + 1) & 1], first, stride, lane);
      if (j + 2 < n_blk) request_block(k_rows, t_chunk + (j + 2) * kGqaBlockKeys, a.T, first, stride, mrow, qd, st);
    }
    const u32x4 *buf = kbuf[j & 1];
    const int t_block = t_chunk + j * kGqaBlockKeys;
    if (t_block + kGqaBlockKeys - 1 <= a.T - a.W) {
      // Every key of the block is seen by every tail row (all but the last blocks of a context): no masks; keys are
      // read from LDS one group ahead of their products, the products issued one group ahead of the exponentials.
      f32x4 acc_a[4], acc_b[4];
      bf16x8 kb_a[4], kb_b[4];
      read_block_group(buf, 0, lane, kb_a);
      read_block_group(buf, 1, lane, kb_b);
      products_of_group<NRB, true>(q, kb_a, acc_a);
#pragma unroll
      for (int g = 0; g < kGqaBlockGroups; g += 2) {
        if (g + 2 < kGqaBlockGroups) read_block_group(buf, g + 2, lane, kb_a);
        products_of_group<NRB, true>(q, kb_b, acc_b);
        stats_add_group<NRB>(st_row, acc_a, scale2, t_block + 16 * g, a.T, a.W, mrow, qd, 16 * rb0);
        if (g + 2 < kGqaBlockGroups) {
          read_block_group(buf, g + 3, lane, kb_b);
          products_of_group<NRB, true>(q, kb_a, acc_a);
        }
        stats_add_group<NRB>(st_row, acc_b, scale2, t_block + 16 * g + 16, a.T, a.W, mrow, qd, 16 * rb0);
      }
    } else {
      for (int g = 0; g < kGqaBlockGroups; ++g) {
        const int t_first = t_block + 16 * g;
        if (t_first >= a.T) break;  // uniform over the workgroup
        f32x4 acc[4];
        score_block_group<NRB, true>(q, buf, g, lane, acc);
        stats_raise_and_add<NRB>(st_row, acc, scale2, t_first, a.T, a.W, mrow, qd, 16 * rb0);
      }
    }
    __syncthreads();
  }
  // this wavefront saw every key of the chunk for its rows: its statistics are the chunk's
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) {
    const float lr = stats_row_sum(st_row.l[rb]);
    if (qd == 0) {
      float *dst = a.row_stats + (((size_t)bhq * a.n_chunk + chunk) * a.W + 16 * (rb0 + rb) + mrow) * 2;
      dst[0] = st_row.m[rb];
      dst[1] = lr;
    }
  }
}

// pass 2: per (b, hkv, chunk): mass[t] = sum over the group's heads and the tail rows of 2^(s - m_row) / l_row (added
// up in wavefront order, i.e. head by head, lower rows first)
template <int NRB, int MAXIT>
__global__ __launch_bounds__(64 * kGqaMaxHeads * (4 / NRB)) void psa_mass_gqa_kernel(SelectArgs a) {
  constexpr int kHeadWaves = 4 / NRB;                      // wavefronts per query head
  constexpr int kMaxWaves = kGqaMaxHeads * kHeadWaves;     // scoring wavefronts of a workgroup, at most
  __shared__ u32x4 kbuf[2][kGqaItems * 64];
  __shared__ float stat_m[kGqaMaxHeads][64], stat_il[kGqaMaxHeads][64];
  // column sums of a block: one slot per (scoring wavefront, row quarter, key), each written by one lane; two copies,
  // so that a block's slots are added up (fixed order) while the next block is being scored
  __shared__ float col_lds[2][kMaxWaves][4][kGqaBlockKeys];
  const int chunk = blockIdx.x, bh = blockIdx.y;
  const int R = a.Hq / a.Hkv, b = bh / a.Hkv, hkv = bh % a.Hkv;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6), lane = threadIdx.x & 63, mrow = lane & 15, qd = lane >> 4;
  const int n_score = R * kHeadWaves;
  const int head = wave / kHeadWaves, rb0 = (wave % kHeadWaves) * NRB;
  const int bhq = b * a.Hq + hkv * R + head;
  const uint16_t *k_rows = a.k + (size_t)bh * a.T * kD;
  const float scale2 = a.sm_scale * kLog2e;
  const int t_chunk = chunk * kScoreChunk;
  const int n_blk = min(kGqaBlocks, (a.T - t_chunk + kGqaBlockKeys - 1) / kGqaBlockKeys);
  // feeders (kGqaItems / MAXIT wavefronts behind the scoring ones) take consecutive pieces; without feeders the
  // scoring wavefronts take pieces wave, wave + kMaxWaves, ...
  constexpr bool kFeeder = MAXIT >= kGqaFeederItems;
  const int first = kFeeder ? (wave - n_score) * MAXIT : wave, stride = kFeeder ? 1 : kMaxWaves;
  // adds up the slots of key `key` of block j (scoring wavefronts in order, quarters pairwise) and stores its mass
  auto flush_key = [&](int j, int key) {
    const int t = t_chunk + j * kGqaBlockKeys + key;
    float sum = 0.0f;
    for (int w = 0; w < n_score; ++w)
      sum += (col_lds[j & 1][w][0][key] + col_lds[j & 1][w][1][key]) +
             (col_lds[j & 1][w][2][key] + col_lds[j & 1][w][3][key]);
    if (t < a.T) a.mass[(size_t)bh * a.T + t] = sum;
  };
  KeyStage<MAXIT> st;
  if (kFeeder && wave >= n_score) {  // a feeder: same barriers as the scoring wavefronts below
    // the feeders share the keys of a block when its column sums are added up
    constexpr int kFeederKeys = kFeeder ? kGqaBlockKeys * MAXIT / kGqaItems : kGqaBlockKeys;
    const int first_key = (wave - n_score) * kFeederKeys;
    request_block(k_rows, t_chunk, a.T, first, stride, mrow, qd, st);
    deposit_block(st, kbuf[0], first, stride, lane);
    request_block(k_rows, t_chunk + kGqaBlockKeys, a.T, first, stride, mrow, qd, st);
    __syncthreads();
    for (int j = 0; j < n_blk; ++j) {
      if (j + 1 < n_blk) deposit_block(st, kbuf[(j + 1) & 1], first, stride, lane);
      if (j + 2 < n_blk) request_block(k_rows, t_chunk + (j + 2) * kGqaBlockKeys, a.T, first, stride, mrow, qd, st);
      if (j > 0 && lane < kFeederKeys) flush_key(j - 1, first_key + lane);
      __syncthreads();
    }
    if (lane < kFeederKeys) flush_key(n_blk - 1, first_key + lane);
    return;
  }
  if constexpr (!kFeeder) request_block(k_rows, t_chunk, a.T, first, stride, mrow, qd, st);
  if (lane < 16 * NRB) {  // merge the chunk statistics of this wavefront's rows
    const int row = 16 * rb0 + lane;
    const float *src = a.row_stats + ((size_t)bhq * a.n_chunk * a.W + row) * 2;
    float mm = -INFINITY;
    for (int c = 0; c < a.n_chunk; ++c) mm = fmaxf(mm, src[(size_t)c * a.W * 2]);
    float ll = 0.0f;
    for (int c = 0; c < a.n_chunk; ++c) {
      const float mc = src[(size_t)c * a.W * 2];
      if (mc != -INFINITY) ll += src[(size_t)c * a.W * 2 + 1] * fast_exp2(mc - mm);
    }
    stat_m[head][row] = mm;
    stat_il[head][row] = 1.0f / ll;
  }
  bf16x8 q[NRB * 4];
  load_query_rows<NRB>(a.q_tail + (size_t)bhq * a.W * kD, rb0, mrow, qd, q);
  if constexpr (!kFeeder) {
    deposit_block(st, kbuf[0], first, stride, lane);
    request_block(k_rows, t_chunk + kGqaBlockKeys, a.T, first, stride, mrow, qd, st);
  }
  wave_lds_sync();  // the statistics read below were written by this wavefront
  f32x4 rm[NRB], ril[NRB];  // rows 16*(rb0 + rb) + 4*qd + i
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) {
    rm[rb] = *reinterpret_cast<const f32x4 *>(&stat_m[head][16 * (rb0 + rb) + 4 * qd]);
    ril[rb] = *reinterpret_cast<const f32x4 *>(&stat_il[head][16 * (rb0 + rb) + 4 * qd]);
  }
  __syncthreads();
  for (int j = 0; j < n_blk; ++j) {
    if constexpr (!kFeeder) {
      if (j + 1 < n_blk) deposit_block(st, kbuf[(j + 1) & 1], first, stride, lane);
      if (j + 2 < n_blk) request_block(k_rows, t_chunk + (j + 2) * kGqaBlockKeys, a.T, first, stride, mrow, qd, st);
      if (j > 0 && threadIdx.x < kGqaBlockKeys) flush_key(j - 1, threadIdx.x);
    }
    const u32x4 *buf = kbuf[j & 1];
    const int t_block = t_chunk + j * kGqaBlockKeys;
    if (t_block + kGqaBlockKeys - 1 <= a.T - a.W) {
      // Every key of the block is seen by every tail row (all but the last blocks of a context): straight-line code,
      // keys read from LDS one group ahead of their products, the products issued one group ahead of the exponentials.
      f32x4 acc[2][4];
      bf16x8 kb[2][4];
      read_block_group(buf, 0, lane, kb[0]);
      read_block_group(buf, 1, lane, kb[1]);
      products_of_group<NRB, false>(q, kb[0], acc[0]);
#pragma unroll
      for (int g = 0; g < kGqaBlockGroups; ++g) {
        const f32x4(&cur)[4] = acc[g & 1];
        if (g + 2 < kGqaBlockGroups) read_block_group(buf, g + 2, lane, kb[g & 1]);
        if (g + 1 < kGqaBlockGroups) products_of_group<NRB, false>(q, kb[(g + 1) & 1], acc[(g + 1) & 1]);
        float c0 = 0.0f, c1 = 0.0f;  // two chains: even and odd row blocks
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb) {
          float &cc = (rb & 1) ? c1 : c0;
#pragma unroll
          for (int i = 0; i < 4; ++i)
            cc = __builtin_fmaf(fast_exp2(__builtin_fmaf(cur[rb][i], scale2, -rm[rb][i])), ril[rb][i], cc);
        }
        col_lds[j & 1][wave][qd][16 * g + mrow] = c0 + c1;
      }
    } else {
      for (int g = 0; g < kGqaBlockGroups; ++g) {
        const int t_first = t_block + 16 * g;
        float c = 0.0f;
        if (t_first < a.T) {  // uniform over the workgroup; groups past the end leave zeros in their slots
          f32x4 acc[4];
          score_block_group<NRB, false>(q, buf, g, lane, acc);
          float c0 = 0.0f, c1 = 0.0f;
          const int t = t_first + mrow;
#pragma unroll
          for (int rb = 0; rb < NRB; ++rb) {
            float &cc = (rb & 1) ? c1 : c0;
#pragma unroll
            for (int i = 0; i < 4; ++i)
              if (key_seen(t, 16 * (rb0 + rb) + 4 * qd + i, a.T, a.W))
                cc = __builtin_fmaf(fast_exp2(__builtin_fmaf(acc[rb][i], scale2, -rm[rb][i])), ril[rb][i], cc);
          }
          c = c0 + c1;
        }
        col_lds[j & 1][wave][qd][16 * g + mrow] = c;
      }
    }
    __syncthreads();
  }
  if constexpr (!kFeeder)
    if (threadIdx.x < kGqaBlockKeys) flush_key(n_blk - 1, threadIdx.x);
}

// inclusive prefix sum of one int per thread over a workgroup of NW wavefronts, plus the workgroup total
template <int NW>
__device__ __forceinline__ int block_inclusive_scan(int v, int *wave_tot, int &total) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int off = 1; off < kWave; off <<= 1) {
    const int up = __shfl_up(v, off, kWave);
    if (lane >= off) v += up;
  }
  __syncthreads();  // previous use of wave_tot finished
  if (lane == kWave - 1) wave_tot[wave] = v;
  __syncthreads();
  int before = 0, tot = 0;
#pragma unroll
  for (int w = 0; w < NW; ++w) {
    const int c = wave_tot[w];
    if (w < wave) before += c;
    tot += c;
  }
  total = tot;
  return before + v;
}

// exact top-k of non-negative fp32 keys by radix select; equal keys go to the lower position; output ascending.
// STAGED: the row of keys is copied to LDS once and every pass reads it from there.
constexpr int kTopkStageMax = 32768;  // keys (128 KB of LDS)
constexpr int kTopkListMax = 256;     // selected positions ordered through LDS when k is at most this
constexpr int kTopkCandMax = 512;     // candidates the short cut ranks among themselves
constexpr int kTopkWideFrom = 8192, kTopkWideRows = 512, kTopkWideThreads = 1024;  // see launch_topk
// NT threads per workgroup (256, or 1024 for long rows: the passes over the keys are what takes the time there)
template <bool STAGED, int NT>
__global__ __launch_bounds__(NT) void topk_kernel(SelectArgs a) {
  extern __shared__ float keys_lds[];
  __shared__ int hist[256];
  __shared__ int wave_tot[NT / 64];
  __shared__ uint32_t sh_prefix;
  __shared__ int sh_need;
  __shared__ int list_n;
  __shared__ int list[kTopkListMax];
  __shared__ uint32_t thread_max[NT];
  __shared__ int cand_n;
  __shared__ uint32_t cand_key[kTopkCandMax];
  __shared__ int cand_pos[kTopkCandMax];
  const int bh = blockIdx.x, lane = threadIdx.x & 63;
  const float *mass = a.mass + (size_t)(a.mass_per_batch ? bh / a.Hkv : bh) * a.T;
  int32_t *out = a.sal_idx + (size_t)bh * a.S_cap;
  const int k = min(a.top_k, a.T);
  const uint32_t lowest = a.skip_zero ? 1u : 0u;  // keys below this bit pattern (i.e. +0) are never selected
  if (STAGED) {
    uint32_t mine = 0u;  // largest key this thread staged (bit patterns of non-negative floats order like the floats)
    for (int t = threadIdx.x; t < a.T; t += NT) {
      const float x = mass[t];
      keys_lds[t] = x;
      mine = max(mine, __float_as_uint(x));
    }
    if (threadIdx.x == 0) { list_n = 0; cand_n = 0; }
    thread_max[threadIdx.x] = mine;
    __syncthreads();
    if (k <= 128) {
      // Short cut for the usual case (a few pivots out of thousands of keys): the k-th largest of the per-thread
      // maxima is a lower bound of the k-th largest key, and few keys reach it.  They are collected and ranked among
      // themselves (key descending, position ascending: the order of the radix path).  Too many candidates (many equal
      // keys): the radix passes below take over.  Every wavefront finds the bound for itself, bit by bit from the top:
      // the largest x with at least k of 256 maxima >= x (four per lane; with more than 256 threads each is the
      // largest of NT / 256 thread maxima, still 256 different keys).
      uint32_t mx[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        uint32_t v = 0u;
#pragma unroll
        for (int jj = 0; jj < NT / 256; ++jj) v = max(v, thread_max[lane + 64 * i + 256 * jj]);
        mx[i] = v;
      }
      uint32_t bound = 0u;
      for (int bit = 31; bit >= 0; --bit) {
        const uint32_t cand = bound | (1u << bit);
        const int n_ge = __popcll(__ballot(mx[0] >= cand)) + __popcll(__ballot(mx[1] >= cand)) +
                         __popcll(__ballot(mx[2] >= cand)) + __popcll(__ballot(mx[3] >= cand));
        if (n_ge >= k) bound = cand;
      }
      for (int t = threadIdx.x; t < a.T; t += NT) {
        const uint32_t bits = __float_as_uint(keys_lds[t]);
        if (bits >= bound && bits >= lowest) {
          const int at = atomicAdd(&cand_n, 1);
          if (at < kTopkCandMax) { cand_key[at] = bits; cand_pos[at] = t; }
        }
      }
      __syncthreads();
      const int n_cand = cand_n;
      if (n_cand <= kTopkCandMax) {  // uniform
        for (int c = threadIdx.x; c < n_cand; c += NT) {
          const uint32_t key = cand_key[c];
          const int pos = cand_pos[c];
          int beaten_by = 0;
          for (int j = 0; j < n_cand; ++j) beaten_by += (cand_key[j] > key) || (cand_key[j] == key && cand_pos[j] < pos);
          if (beaten_by < k) list[atomicAdd(&list_n, 1)] = pos;
        }
        __syncthreads();
        const int n_kept = list_n;  // k, or fewer when zero keys are excluded
        if ((int)threadIdx.x < n_kept) {
          const int mine_pos = list[threadIdx.x];
          int rank = 0;
          for (int j = 0; j < n_kept; ++j) rank += list[j] < mine_pos;
          if (rank < a.S_cap) out[rank] = mine_pos;
        }
        if (threadIdx.x == 0) a.sal_cnt[bh] = n_kept;
        return;
      }
      __syncthreads();
      if (threadIdx.x == 0) list_n = 0;
      __syncthreads();
    }
  }
  const float *keys = STAGED ? keys_lds : mass;
  uint32_t prefix = 0;
  int need = k;
  for (int pass = 3; pass >= 0; --pass) {
    if (threadIdx.x < 256) hist[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t hi_mask = pass == 3 ? 0u : (0xFFFFFFFFu << (8 * (pass + 1)));
    for (int t = threadIdx.x; t < a.T; t += NT) {
      const uint32_t bits = __float_as_uint(keys[t]);
      if ((bits & hi_mask) == (prefix & hi_mask)) {
        // the leading digits of the keys of a wavefront mostly coincide: one add for all of them then
        const int bin = (bits >> (8 * pass)) & 0xFF;
        const int first = __builtin_amdgcn_readfirstlane(bin);
        const unsigned long long active = __ballot(true), same = __ballot(bin == first);
        if (same == active) {
          if (lane == __ffsll((long long)active) - 1) atomicAdd(&hist[first], __popcll(active));
        } else {
          atomicAdd(&hist[bin], 1);
        }
      }
    }
    __syncthreads();
    // thread i looks at bin 255-i: the prefix sum over threads is the count of candidates in bins >= that bin; the
    // digit of the k-th largest key is the first bin (from the top) where that count reaches `need`
    const int bin = 255 - (int)threadIdx.x;  // (threads past the 256 bins add nothing to the sums)
    const int mine = bin >= 0 ? hist[bin] : 0;
    int total;
    const int upto = block_inclusive_scan<NT / 64>(mine, wave_tot, total);
    if (bin >= 0 && upto >= need && upto - mine < need) {
      sh_prefix = prefix | ((uint32_t)bin << (8 * pass));
      sh_need = need - (upto - mine);
      if (pass == 0) hist[0] = mine;  // number of keys equal to the k-th largest (bin 0's own count is not needed again)
    }
    __syncthreads();
    prefix = sh_prefix;
    need = sh_need;
  }
  // prefix = bit pattern of the k-th largest key; `need` of the keys equal to it are taken, lowest positions first.
  const int n_equal = hist[0];
  if (STAGED && k <= kTopkListMax && n_equal == need) {
    // every key >= prefix is taken: gather their positions in any order, then order the short list by rank
    for (int t = threadIdx.x; t < a.T; t += NT) {
      const uint32_t bits = __float_as_uint(keys[t]);
      if (bits >= prefix && bits >= lowest) list[atomicAdd(&list_n, 1)] = t;
    }
    __syncthreads();
    const int n_kept = list_n;  // k, or fewer when zero keys are excluded
    if ((int)threadIdx.x < n_kept) {
      const int mine = list[threadIdx.x];
      int rank = 0;
      for (int j = 0; j < n_kept; ++j) rank += list[j] < mine;
      if (rank < a.S_cap) out[rank] = mine;
    }
    if (threadIdx.x == 0) a.sal_cnt[bh] = n_kept;
    return;
  }
  // general case: each thread owns a contiguous run of positions, so two workgroup scans (equal keys, taken keys)
  // order the output
  const int per = (a.T + NT - 1) / NT;
  const int t0 = min((int)threadIdx.x * per, a.T), t1 = min(t0 + per, a.T);
  int n_eq = 0;
  for (int t = t0; t < t1; ++t) n_eq += __float_as_uint(keys[t]) == prefix;
  int tot_eq;
  int eq_rank = block_inclusive_scan<NT / 64>(n_eq, wave_tot, tot_eq) - n_eq;
  int n_take = 0;
  {
    int r = eq_rank;
    for (int t = t0; t < t1; ++t) {
      const uint32_t bits = __float_as_uint(keys[t]);
      n_take += (bits > prefix || (bits == prefix && r++ < need)) && bits >= lowest;
    }
  }
  int tot_take;
  int pos = block_inclusive_scan<NT / 64>(n_take, wave_tot, tot_take) - n_take;
  if (n_take > 0) {
    for (int t = t0; t < t1; ++t) {
      const uint32_t bits = __float_as_uint(keys[t]);
      if ((bits > prefix || (bits == prefix && eq_rank++ < need)) && bits >= lowest) {
        if (pos < a.S_cap) out[pos] = t;
        ++pos;
      }
    }
  }
  if (threadIdx.x == 0) a.sal_cnt[bh] = tot_take;
}

// ---- massive-activation score (Section III-B.2): largest channel magnitude of every token's hidden state ----
// One wavefront per token; magnitudes of binary16 values order like their low 15 bits, so the row maximum is taken on
// integers; scores below the floor are written as 0 (the top-k never selects a zero key).
__global__ __launch_bounds__(256) void massive_score_kernel(SelectArgs a) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const long row = (long)blockIdx.x * 4 + wave;
  if (row >= (long)a.B * a.T) return;
  const uint16_t *src = a.hidden + (size_t)row * a.d_model;
  uint32_t m0 = 0u, m1 = 0u;  // running maxima of the low and the high binary16 of every word, as 15-bit integers
  for (int c0 = 0; c0 < a.d_model; c0 += 512) {  // 64 lanes x 8 channels
    const u32x4 v = stream_load(reinterpret_cast<const u32x4 *>(src + c0 + 8 * lane));
    const uint32_t w0 = v[0], w1 = v[1], w2 = v[2], w3 = v[3];
    m0 = max(m0, max(max(w0 & 0x7FFFu, w1 & 0x7FFFu), max(w2 & 0x7FFFu, w3 & 0x7FFFu)));
    m1 = max(m1, max(max((w0 >> 16) & 0x7FFFu, (w1 >> 16) & 0x7FFFu), max((w2 >> 16) & 0x7FFFu, (w3 >> 16) & 0x7FFFu)));
  }
  uint32_t m2 = max(m0, m1);
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) m2 = max(m2, (uint32_t)__shfl_xor((int)m2, off, kWave));
  if (lane == 0) {
    const float score = half_bits_to_float(m2);
    a.mass[row] = score >= a.floor ? score : 0.0f;
  }
}

}  // namespace

// Dynamic LDS above 48 KB has to be opted into, per device and process: done on the first launch that needs it on a
// device (for the largest size the kernel is ever given), not on every call.
static hipError_t topk_allow_large_lds() {
  static std::atomic<unsigned long long> done{0};
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev >= 0 && dev < 64 && ((done.load(std::memory_order_acquire) >> dev) & 1ull)) return hipSuccess;
  e = hipFuncSetAttribute(reinterpret_cast<const void *>(&topk_kernel<true, kTopkWideThreads>),
                          hipFuncAttributeMaxDynamicSharedMemorySize, (int)(kTopkStageMax * sizeof(float)));
  if (e == hipSuccess)
    e = hipFuncSetAttribute(reinterpret_cast<const void *>(&topk_kernel<true, 256>),
                            hipFuncAttributeMaxDynamicSharedMemorySize, (int)(kTopkStageMax * sizeof(float)));
  if (e == hipSuccess && dev >= 0 && dev < 64) done.fetch_or(1ull << dev, std::memory_order_release);
  return e;
}

// One workgroup per row of keys.  Few long rows (at most kTopkWideRows rows of kTopkWideFrom keys or more) get
// workgroups of 1024 threads: the time goes into the passes over the keys then, and 256-thread workgroups would leave
// most of the chip idle.  With many rows the small workgroups already fill it (and are 6 % faster at 2048 x 8192).
static hipError_t launch_topk(const SelectArgs &k, hipStream_t stream) {
  const dim3 grid(k.B * k.Hkv);
  const bool wide = k.T >= kTopkWideFrom && (long)k.B * k.Hkv <= kTopkWideRows;
  const size_t lds = k.T <= kTopkStageMax ? (size_t)k.T * sizeof(float) : 0;
  if (lds > 48 * 1024) {
    hipError_t e = topk_allow_large_lds();
    if (e != hipSuccess) return e;
  }
  if (k.T > kTopkStageMax) {
    if (wide) hipLaunchKernelGGL((topk_kernel<false, kTopkWideThreads>), grid, dim3(kTopkWideThreads), 0, stream, k);
    else hipLaunchKernelGGL((topk_kernel<false, 256>), grid, dim3(256), 0, stream, k);
  } else {
    if (wide) hipLaunchKernelGGL((topk_kernel<true, kTopkWideThreads>), grid, dim3(kTopkWideThreads), lds, stream, k);
    else hipLaunchKernelGGL((topk_kernel<true, 256>), grid, dim3(256), lds, stream, k);
  }
  return hipGetLastError();
}

hipError_t launch_select_massive(const SelectArgs &a, hipStream_t stream) {
  const long rows = (long)a.B * a.T;
  hipLaunchKernelGGL(massive_score_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, stream, a);
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  return launch_topk(a, stream);
}

hipError_t launch_select_tsa(const SelectArgs &a, hipStream_t stream) {
  hipLaunchKernelGGL(select_tsa_kernel, dim3(a.B * a.Hkv), dim3(256), 0, stream, a);
  return hipGetLastError();
}

namespace {

// token-level pivots: the masses of a batch element's kv-heads added in head order (one thread per position)
__global__ __launch_bounds__(256) void sum_heads_kernel(SelectArgs a) {
  const long i = (long)blockIdx.x * 256 + threadIdx.x;
  if (i >= (long)a.B * a.T) return;
  const int b = (int)(i / a.T), t = (int)(i % a.T);
  float sum = 0.0f;
  for (int h = 0; h < a.Hkv; ++h) sum += a.mass[((size_t)b * a.Hkv + h) * a.T + t];
  a.mass_shared[i] = sum;
}

}  // namespace

// FEEDER: fewer than eight heads per KV head (room for feeder wavefronts behind the scoring ones)
template <bool FEEDER>
static void launch_psa_gqa_passes(const SelectArgs &a, hipStream_t stream) {
  const int R = a.Hq / a.Hkv;
  const dim3 grid(a.n_chunk, a.B * a.Hkv);
  // first pass: two wavefronts per head and two feeders (one feeder would be the slowest wavefront of the workgroup:
  // about 240 vector instructions per block against 150 of a scoring wavefront); second pass: one per head, one feeder
  hipLaunchKernelGGL((psa_row_stats_gqa_kernel<2, FEEDER ? kGqaItems / 2 : kGqaItems / (2 * kGqaMaxHeads)>), grid,
                     dim3(64 * (2 * R + (FEEDER ? 2 : 0))), 0, stream, a);
  if (R == 1) {
    // one head: a single scoring wavefront would leave the workgroup at two wavefronts; two of 32 rows and two feeders
    hipLaunchKernelGGL((psa_mass_gqa_kernel<2, kGqaItems / 2>), grid, dim3(64 * 4), 0, stream, a);
    return;
  }
  // (two wavefronts per head and two feeders, measured with seven heads: 692 against 645 us at cfg5)
  hipLaunchKernelGGL((psa_mass_gqa_kernel<4, FEEDER ? kGqaItems : kGqaItems / kGqaMaxHeads>), grid,
                     dim3(64 * (R + (FEEDER ? 1 : 0))), 0, stream, a);
}
template <int NRB>
static void launch_psa_passes(const SelectArgs &a, hipStream_t stream) {
  if constexpr (NRB == 4) {  // the kernels with feeder wavefronts exist for W = 64 only
    const int R = a.Hq / a.Hkv;
    if (R == kGqaMaxHeads) return launch_psa_gqa_passes<false>(a, stream);
    if (R >= 1 && R < kGqaMaxHeads) return launch_psa_gqa_passes<true>(a, stream);
  }
  const dim3 block(256);
  hipLaunchKernelGGL(psa_row_stats_kernel<NRB>, dim3(a.n_chunk, a.B * a.Hq), block, 0, stream, a);
  hipLaunchKernelGGL(psa_mass_kernel<NRB>, dim3(a.n_chunk, a.B * a.Hkv), block, 0, stream, a);
}

hipError_t launch_select_psa(const SelectArgs &a, hipStream_t stream) {
  switch (a.W / 16) {
    case 1: launch_psa_passes<1>(a, stream); break;
    case 2: launch_psa_passes<2>(a, stream); break;
    case 3: launch_psa_passes<3>(a, stream); break;
    default: launch_psa_passes<4>(a, stream); break;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  SelectArgs k = a;  // what the top-k reads
  if (a.mass_shared != nullptr) {
    hipLaunchKernelGGL(sum_heads_kernel, dim3((unsigned)(((long)a.B * a.T + 255) / 256)), dim3(256), 0, stream, a);
    e = hipGetLastError();
    if (e != hipSuccess) return e;
    k.mass = a.mass_shared;
    k.mass_per_batch = 1;
  }
  return launch_topk(k, stream);
}

}  // namespace akvq

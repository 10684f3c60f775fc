// Salient-token identification (Section III-B of arXiv 2501.15021).
//   TSA layers: the salient set is the text positions -> ordered stream compaction of the modality mask.
//   PSA layers: pivot tokens are the few tokens that receive most of the attention (Section I / III-A.3); the score
//   is the attention-column mass of the last W prompt rows, computed on the matrix cores (bfloat16 operands, fp32
//   accumulate, fp32 softmax) in two streaming passes over K (row statistics, then column sums), followed by an
//   exact top-k (radix select on the fp32 bit patterns, ties to the lower position).
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
// Each workgroup (4 wavefronts) owns kScoreChunk consecutive keys of one (batch, head); a wavefront walks its quarter
// in groups of 16 keys, with the next group's loads in flight while the current one goes through the matrix cores.
// Logits are kept in the base-2 domain (sm_scale * log2(e) folded into one multiply) so that exponentials are bare
// v_exp_f32; both passes use the same domain, so the statistics carry over unchanged.
constexpr int kGroupsPerWave = kScoreChunk / (4 * 16);

// binary16 pair (packed) -> bfloat16 pair (packed), each rounded to nearest even
__device__ __forceinline__ uint32_t half2_to_bf16x2(uint32_t hh) {
  return pack_bf16x2(half_bits_to_float(hh & 0xFFFFu), half_bits_to_float(hh >> 16));
}
__device__ __forceinline__ bf16x8 rows8_as_bf16(u32x4 raw) {
  u32x4 r = {half2_to_bf16x2(raw[0]), half2_to_bf16x2(raw[1]), half2_to_bf16x2(raw[2]), half2_to_bf16x2(raw[3])};
  return __builtin_bit_cast(bf16x8, r);
}
__device__ __forceinline__ float row_max16(float v) {
#pragma unroll
  for (int off = 8; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
  return v;
}
__device__ __forceinline__ float row_sum16(float v) {
#pragma unroll
  for (int off = 8; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

struct KeyGroup {
  u32x4 raw[4];  // 16 keys x 128 channels as this lane's four 8-channel pieces (binary16)
};
__device__ __forceinline__ void load_key_group(const uint16_t *k_rows, int t_first, int T, int mrow, int qd, KeyGroup &g) {
  const int t = t_first + mrow;
#pragma unroll
  for (int kc = 0; kc < 4; ++kc) {
    if (t < T) g.raw[kc] = *reinterpret_cast<const u32x4 *>(k_rows + (size_t)t * kD + 32 * kc + 8 * qd);
    else g.raw[kc] = (u32x4){0u, 0u, 0u, 0u};
  }
}

// base-2 logits of the W tail rows of one query head against 16 keys: s[rb][i] = row 16*rb + 4*qd + i, key = mrow.
// Entries the causal mask removes (or keys beyond T) come back as -inf.
template <int NRB>
__device__ __forceinline__ void score_16keys(const bf16x8 (&a_q)[4][4], const KeyGroup &g, int t_first, int T, int W,
                                             float scale2, int mrow, int qd, float (&s)[4][4]) {
  const int t = t_first + mrow;
  bf16x8 kb[4];
#pragma unroll
  for (int kc = 0; kc < 4; ++kc) kb[kc] = rows8_as_bf16(g.raw[kc]);
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb) {
    f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int kc = 0; kc < 4; ++kc) acc = mfma_bf16(a_q[rb][kc], kb[kc], acc);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const int row = 16 * rb + 4 * qd + i;
      const bool seen = t < T && t <= T - W + row;  // causal: row sits at position T-W+row
      s[rb][i] = seen ? scale2 * acc[i] : -INFINITY;
    }
  }
}

template <int NRB>
__device__ __forceinline__ void load_query_rows(const uint16_t *q_head, int mrow, int qd, bf16x8 (&a_q)[4][4]) {
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
    for (int kc = 0; kc < 4; ++kc)
      a_q[rb][kc] = rows8_as_bf16(
          *reinterpret_cast<const u32x4 *>(q_head + (size_t)(16 * rb + mrow) * kD + 32 * kc + 8 * qd));
}

constexpr float kLog2e = 1.4426950408889634f;
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }  // bare v_exp_f32

// pass 1: per (b, hq, chunk): running max and sum of exponentials (base 2) of every tail row
template <int NRB>
__global__ __launch_bounds__(256) void psa_row_stats_kernel(SelectArgs a) {
  __shared__ float st_m[4][64], st_l[4][64];
  const int chunk = blockIdx.x, bhq = blockIdx.y;
  const int b = bhq / a.Hq, hq = bhq % a.Hq, hkv = hq / (a.Hq / a.Hkv);
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, mrow = lane & 15, qd = lane >> 4;
  const uint16_t *k_rows = a.k + ((size_t)b * a.Hkv + hkv) * a.T * kD;
  const float scale2 = a.sm_scale * kLog2e;
  bf16x8 a_q[4][4];
  load_query_rows<NRB>(a.q_tail + (size_t)bhq * a.W * kD, mrow, qd, a_q);
  float m[4][4], l[4][4];
#pragma unroll
  for (int rb = 0; rb < 4; ++rb)
#pragma unroll
    for (int i = 0; i < 4; ++i) { m[rb][i] = -INFINITY; l[rb][i] = 0.0f; }
  const int t_wave = chunk * kScoreChunk + wave * (kScoreChunk / 4);
  KeyGroup cur, nxt;
  load_key_group(k_rows, t_wave, a.T, mrow, qd, cur);
#pragma unroll
  for (int kc = 0; kc < 4; ++kc) settle(cur.raw[kc]);
  for (int g = 0; g < kGroupsPerWave; ++g) {
    const int t_first = t_wave + 16 * g;
    if (t_first >= a.T) break;
    if (g + 1 < kGroupsPerWave) load_key_group(k_rows, t_first + 16, a.T, mrow, qd, nxt);
    float s[4][4];
    score_16keys<NRB>(a_q, cur, t_first, a.T, a.W, scale2, mrow, qd, s);
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const float m_new = fmaxf(m[rb][i], s[rb][i]);
        const float m_ref = (m_new == -INFINITY) ? 0.0f : m_new;
        l[rb][i] = l[rb][i] * fast_exp2(m[rb][i] - m_ref) + fast_exp2(s[rb][i] - m_ref);
        m[rb][i] = m_new;
      }
    cur = nxt;
  }
#pragma unroll
  for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      const float mr = row_max16(m[rb][i]);
      const float m_ref = (mr == -INFINITY) ? 0.0f : mr;
      const float lr = row_sum16(l[rb][i] * fast_exp2(m[rb][i] - m_ref));
      if (mrow == 0) { st_m[wave][16 * rb + 4 * qd + i] = mr; st_l[wave][16 * rb + 4 * qd + i] = lr; }
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
__global__ __launch_bounds__(256) void psa_mass_kernel(SelectArgs a) {
  __shared__ float row_m[64], row_il[64];
  const int chunk = blockIdx.x, bh = blockIdx.y;
  const int b = bh / a.Hkv, hkv = bh % a.Hkv, R = a.Hq / a.Hkv;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63, mrow = lane & 15, qd = lane >> 4;
  const uint16_t *k_rows = a.k + (size_t)bh * a.T * kD;
  const float scale2 = a.sm_scale * kLog2e;
  const int t_wave = chunk * kScoreChunk + wave * (kScoreChunk / 4);
  float col[kGroupsPerWave];
#pragma unroll
  for (int g = 0; g < kGroupsPerWave; ++g) col[g] = 0.0f;
  for (int h = 0; h < R; ++h) {
    const int bhq = b * a.Hq + hkv * R + h;
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
    __syncthreads();
    bf16x8 a_q[4][4];
    load_query_rows<NRB>(a.q_tail + (size_t)bhq * a.W * kD, mrow, qd, a_q);
    float rm[4][4], ril[4][4];
#pragma unroll
    for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
      for (int i = 0; i < 4; ++i) { rm[rb][i] = row_m[16 * rb + 4 * qd + i]; ril[rb][i] = row_il[16 * rb + 4 * qd + i]; }
    KeyGroup cur, nxt;
    load_key_group(k_rows, t_wave, a.T, mrow, qd, cur);
#pragma unroll
    for (int kc = 0; kc < 4; ++kc) settle(cur.raw[kc]);
#pragma unroll
    for (int g = 0; g < kGroupsPerWave; ++g) {
      const int t_first = t_wave + 16 * g;
      if (t_first < a.T) {  // uniform over the wavefront
        if (g + 1 < kGroupsPerWave) load_key_group(k_rows, t_first + 16, a.T, mrow, qd, nxt);
        float s[4][4];
        score_16keys<NRB>(a_q, cur, t_first, a.T, a.W, scale2, mrow, qd, s);
#pragma unroll
        for (int rb = 0; rb < NRB; ++rb)
#pragma unroll
          for (int i = 0; i < 4; ++i) col[g] += fast_exp2(s[rb][i] - rm[rb][i]) * ril[rb][i];  // 2^-inf = 0 for masked
        cur = nxt;
      }
    }
  }
#pragma unroll
  for (int g = 0; g < kGroupsPerWave; ++g) {
    float c = col[g];
    c += __shfl_xor(c, 16, kWave);
    c += __shfl_xor(c, 32, kWave);
    const int t = t_wave + 16 * g + mrow;
    if (qd == 0 && t < a.T) a.mass[(size_t)bh * a.T + t] = c;
  }
}

// exact top-k of non-negative fp32 keys by radix select; equal keys go to the lower position; output ascending
__global__ __launch_bounds__(256) void topk_kernel(SelectArgs a) {
  __shared__ int hist[256];
  __shared__ int wave_tot[4];
  __shared__ uint32_t sh_prefix;
  __shared__ int sh_need;
  const int bh = blockIdx.x;
  const float *mass = a.mass + (size_t)bh * a.T;
  int32_t *out = a.sal_idx + (size_t)bh * a.S_cap;
  const int k = min(a.top_k, a.T);
  uint32_t prefix = 0;
  int need = k;
  for (int pass = 3; pass >= 0; --pass) {
    hist[threadIdx.x] = 0;
    __syncthreads();
    const uint32_t hi_mask = pass == 3 ? 0u : (0xFFFFFFFFu << (8 * (pass + 1)));
    for (int t = threadIdx.x; t < a.T; t += 256) {
      const uint32_t bits = __float_as_uint(mass[t]);
      if ((bits & hi_mask) == (prefix & hi_mask)) atomicAdd(&hist[(bits >> (8 * pass)) & 0xFF], 1);
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      int remaining = need, bin = 255;
      for (; bin > 0; --bin) {
        if (hist[bin] >= remaining) break;
        remaining -= hist[bin];
      }
      sh_prefix = prefix | ((uint32_t)bin << (8 * pass));
      sh_need = remaining;
    }
    __syncthreads();
    prefix = sh_prefix;
    need = sh_need;
    __syncthreads();
  }
  // prefix = bit pattern of the k-th largest key; `need` of the keys equal to it are taken, lowest positions first
  int n_out = 0, n_equal = 0;
  for (int base = 0; base < a.T; base += 256) {
    const int t = base + threadIdx.x;
    const uint32_t bits = t < a.T ? __float_as_uint(mass[t]) : 0u;
    const bool greater = t < a.T && bits > prefix;
    const bool equal = t < a.T && bits == prefix;
    int tot_eq;
    const int eq_rank = n_equal + block_flag_scan(equal, wave_tot, tot_eq);
    const bool take = greater || (equal && eq_rank < need);
    int tot_take;
    const int pos = n_out + block_flag_scan(take, wave_tot, tot_take);
    if (take && pos < a.S_cap) out[pos] = t;
    n_out += tot_take;
    n_equal += tot_eq;
  }
  if (threadIdx.x == 0) a.sal_cnt[bh] = n_out;
}

}  // namespace

hipError_t launch_select_tsa(const SelectArgs &a, hipStream_t stream) {
  hipLaunchKernelGGL(select_tsa_kernel, dim3(a.B * a.Hkv), dim3(256), 0, stream, a);
  return hipGetLastError();
}

hipError_t launch_select_psa(const SelectArgs &a, hipStream_t stream) {
  const dim3 block(256);
  const dim3 g1(a.n_chunk, a.B * a.Hq), g2(a.n_chunk, a.B * a.Hkv);
  switch (a.W / 16) {
    case 1:
      hipLaunchKernelGGL(psa_row_stats_kernel<1>, g1, block, 0, stream, a);
      hipLaunchKernelGGL(psa_mass_kernel<1>, g2, block, 0, stream, a);
      break;
    case 2:
      hipLaunchKernelGGL(psa_row_stats_kernel<2>, g1, block, 0, stream, a);
      hipLaunchKernelGGL(psa_mass_kernel<2>, g2, block, 0, stream, a);
      break;
    case 3:
      hipLaunchKernelGGL(psa_row_stats_kernel<3>, g1, block, 0, stream, a);
      hipLaunchKernelGGL(psa_mass_kernel<3>, g2, block, 0, stream, a);
      break;
    default:
      hipLaunchKernelGGL(psa_row_stats_kernel<4>, g1, block, 0, stream, a);
      hipLaunchKernelGGL(psa_mass_kernel<4>, g2, block, 0, stream, a);
      break;
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(topk_kernel, dim3(a.B * a.Hkv), dim3(256), 0, stream, a);
  return hipGetLastError();
}

}  // namespace akvq

// Read path of the AKVQ-VL cache: decode attention straight from the packed 2-bit + bfloat16 cache
// (decode step of Section II-A over the cache of Section III-C, arXiv 2501.15021).
//
// A workgroup of four wavefronts owns one (batch, kv-head, KV-split); the wavefronts take its 64-token (MHA) or
// 32-token (GQA) tiles round-robin and merge their partial softmaxes through LDS.  Both contractions run on the
// matrix cores with the 2-bit codes expanded to bfloat16 integers in registers (one and-or per two codes, see
// akvq_device.h):
//   scores  S = Q~ * C_K^T   : rows = the query vector split into bfloat16 terms, K-dim = 128 channels,
//   output  O = W  * C_V     : rows = (softmax weight x scale) split into bfloat16 terms, K-dim = 32 tokens.
// Scale, zero-point and the constants of the expansion are applied to the small side of each product
// (per token for S, per channel-class for O), so the streamed bytes are touched once, by one and-or each.
// The cache block layout makes each lane's 128-bit load its own matrix-core operand: no shuffles.  The next
// tile's loads are issued before the current tile is consumed.
#include <mutex>
#include <type_traits>

#include "akvq_device.h"
#include "akvq_kernels.h"
#include "akvq_rowquant.h"

namespace akvq {

// Split-KV partial results for callers that may not allocate (akvq_decode_attention_static): a fixed array in the
// library's own device image, one copy per GPU, held until the process ends.  In host code this name is only a
// handle; the device address comes from decode_static_scratch() below and is what the kernels are given.
static __device__ __align__(256) unsigned char scratch[kDecodeStaticScratchBytes];

hipError_t decode_static_scratch(void **ptr) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static void *addr[kMaxDevices] = {};
  int dev = -1;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (addr[dev] == nullptr) {  // once per device, with that device current: every GPU has its own copy of the array
    void *p = nullptr;
    e = hipGetSymbolAddress(&p, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (p == nullptr) return hipErrorInvalidSymbol;
    addr[dev] = p;
  }
  *ptr = addr[dev];
  return hipSuccess;
}

namespace {

constexpr int kWaves = 4;  // wavefronts per workgroup

// ------------------------------------------------------------------------------------------------
// Orthonormal 128-point Walsh-Hadamard transform (Section III-C.2) of a vector held by one wavefront, two elements
// per lane: x0 = element `lane`, x1 = element `lane + 64`.  Strides 1..32 exchange lanes, stride 64 stays in the lane.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ void wht128_wave(float &x0, float &x1, int lane) {
#pragma unroll
  for (int h = 1; h < kWave; h *= 2) {
    const float p0 = __shfl_xor(x0, h, kWave), p1 = __shfl_xor(x1, h, kWave);
    x0 = (lane & h) ? p0 - x0 : x0 + p0;
    x1 = (lane & h) ? p1 - x1 : x1 + p1;
  }
  const float s = x0 + x1, d = x0 - x1;
  x0 = s * inv_sqrt128();
  x1 = d * inv_sqrt128();
}
// rotate a query row inside one wavefront (unless it arrives rotated) and leave it in LDS (the caller synchronises before other waves read it)
// A pre-RoPE query (cos_row != null) first takes its rotary position embedding: channel i pairs with i + 64, both held
// by this lane; exact fp32 products, one rounding of their sum to fp32, then to binary16 (kept apart by the barrier).
__device__ __forceinline__ void rotate_query_lds(const uint16_t *q_row, float *qf, bool q_rotated,
                                                 const uint16_t *cos_row, const uint16_t *sin_row, int lane) {
  float x0 = half_bits_to_float(q_row[lane]), x1 = half_bits_to_float(q_row[lane + 64]);
  if (cos_row != nullptr) {
    const float c = half_bits_to_float(cos_row[lane]), sn = half_bits_to_float(sin_row[lane]);
    float r0 = __fmaf_rn(x0, c, -__fmul_rn(x1, sn)), r1 = __fmaf_rn(x1, c, __fmul_rn(x0, sn));
    asm("" : "+v"(r0));
    asm("" : "+v"(r1));
    x0 = half_bits_to_float(float_to_half_bits_rne(r0));
    x1 = half_bits_to_float(float_to_half_bits_rne(r1));
  }
  if (!q_rotated) wht128_wave(x0, x1, lane);
  qf[lane] = x0;
  qf[lane + 64] = x1;
}

// exponent k of the 4^k factor that the expansion attaches to channel e of a K row (see the K block layout:
// channel e sits in code pair e%8 of its word; pairs 0..3 are the X operand, 4..7 the Y operand)
__device__ __forceinline__ int k_channel_exp(int e) { return pair_exp(e & 3); }
// position of channel e inside the 128-entry A-operand image of a K row: MFMA kc = 2*(e/64) + (e%8)/4, lane group
// qd = (e%32)/8, pair i = e%4, element 2i + (e/32)%2
__device__ __forceinline__ int k_operand_pos(int e) {
  const int m = e >> 5, j = (e >> 3) & 3, ie = e & 7;
  const int kc = 2 * (m >> 1) + (ie >> 2);
  return (4 * kc + j) * 8 + 2 * (ie & 3) + (m & 1);
}
// position of channel e inside the 128-byte A-operand image of the int8 score product: word kc = e/64, lane group
// qd = (e%32)/8, code slot s = 8*((e/32)%2) + e%8 -> register j = s%4, byte b = s/4 -> byte 4j + b of the lane's 16
__device__ __forceinline__ int k_digit_pos(int e) {
  const int kc = e >> 6, j_lane = (e >> 3) & 3, slot = 8 * ((e >> 5) & 1) + (e & 7);
  return (4 * kc + j_lane) * 16 + 4 * (slot & 3) + (slot >> 2);
}
__device__ __forceinline__ float pow4_neg(int k) { return k == 0 ? 1.0f : (k == 1 ? 0.25f : 0.0625f); }

__device__ __forceinline__ uint32_t pack16(uint32_t lo, uint32_t hi) { return (lo & 0xFFFFu) | (hi << 16); }
__device__ __forceinline__ uint32_t hi16(float f) { return __float_as_uint(f) >> 16; }

struct Meta {
  float scale, zero;
  bool salient;
};
__device__ __forceinline__ Meta unpack_meta(uint32_t w) {
  Meta m;
  m.scale = __builtin_fabsf(half_bits_to_float(w & 0xFFFFu));  // bit 15 is the salient flag: dropped by the abs modifier
  m.zero = (float)((int)w >> 16);
  m.salient = (w & 0x8000u) != 0;
  return m;
}

// bit 15 of a meta word marks a salient row; read as binary16 the low half is then a negative number (or -0), which one
// class test detects
__device__ __forceinline__ bool meta_is_salient(uint32_t w) {
  return __builtin_amdgcn_classh(__builtin_bit_cast(_Float16, (unsigned short)w), 0x3C | 0x3);  // any negative class or NaN
}
// w minus one bfloat16 of `pair`: pair . sel + w in one dot-product instruction, sel = (-1, 0) or (0, -1) as a bfloat16
// pair held in a register.  Exact: the remainder of a rounding to bfloat16 has at most 16 significant bits.
__device__ __forceinline__ float minus_bf16(uint32_t pair, uint32_t sel, float w) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
  return __builtin_amdgcn_fdot2_f32_bf16(__builtin_bit_cast(bf16x2_t, pair), __builtin_bit_cast(bf16x2_t, sel), w, false);
}

// two-term bfloat16 split, w ~= hi + lo (16 significant bits): hi is w truncated to its upper 16 bits (so storing
// the upper half of the register stores hi), lo is the exactly representable remainder rounded to bfloat16
__device__ __forceinline__ void split2(float w, float &hif, float &lof) {
  hif = __uint_as_float(__float_as_uint(w) & 0xFFFF0000u);
  lof = __uint_as_float(pack_bf16x2(w - hif, 0.0f) << 16);
}
constexpr float kLog2e = 1.4426950408889634f;
constexpr float kLn2 = 0.6931471805599453f;
constexpr float kLazyMax = 12.0f;  // the softmax reference is raised only when a score exceeds it by 2^12
constexpr float kNoScore = -1.0e30f;  // softmax reference of the grouped-query kernel before its first score
__device__ __forceinline__ float fast_exp2(float x) { return __builtin_amdgcn_exp2f(x); }  // bare v_exp_f32

// ---- DPP reductions over the wavefront (result in every lane) ----
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v) {
  return __int_as_float(__builtin_amdgcn_update_dpp(__float_as_int(v), __float_as_int(v), CTRL, 0xF, 0xF, false));
}
__device__ __forceinline__ float lane_bcast(float v, int l) {
  return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}
__device__ __forceinline__ float row_max_dpp(float v) {  // max over each row of 16 lanes
  v = fmaxf(v, dpp_f<0xB1>(v));   // quad_perm [1,0,3,2]
  v = fmaxf(v, dpp_f<0x4E>(v));   // quad_perm [2,3,0,1]
  v = fmaxf(v, dpp_f<0x141>(v));  // row_half_mirror
  v = fmaxf(v, dpp_f<0x140>(v));  // row_mirror
  return v;
}
__device__ __forceinline__ float row_sum_dpp(float v) {
  v += dpp_f<0xB1>(v);
  v += dpp_f<0x4E>(v);
  v += dpp_f<0x141>(v);
  v += dpp_f<0x140>(v);
  return v;
}
__device__ __forceinline__ float wave_max_dpp(float v) {
  v = row_max_dpp(v);
  return fmaxf(fmaxf(lane_bcast(v, 0), lane_bcast(v, 16)), fmaxf(lane_bcast(v, 32), lane_bcast(v, 48)));
}
__device__ __forceinline__ float wave_sum_dpp(float v) {
  v = row_sum_dpp(v);
  return (lane_bcast(v, 0) + lane_bcast(v, 16)) + (lane_bcast(v, 32) + lane_bcast(v, 48));
}

// Final step: `row` (LDS, 128 floats, complete and visible to this wavefront) is the merged, normalised o~; rotate
// it back (H is its own inverse) unless the caller wants it rotated, and store.  One wavefront does the whole row.
// `out` is the output array ([B][Hq][128] fp32, or binary16 when out_half), `row_index` the (batch, query-head) row.
__device__ __forceinline__ void unrotate_store_wave(const float *row, void *out, size_t row_index, bool out_rotated,
                                                    bool out_half, int lane) {
  float x0 = row[lane], x1 = row[lane + 64];
  if (!out_rotated) wht128_wave(x0, x1, lane);
  if (out_half) {
    uint16_t *o = static_cast<uint16_t *>(out) + row_index * kD;
    o[lane] = (uint16_t)float_to_half_bits_rne(x0);
    o[lane + 64] = (uint16_t)float_to_half_bits_rne(x1);
  } else {
    float *o = static_cast<float *>(out) + row_index * kD;
    o[lane] = x0;
    o[lane + 64] = x1;
  }
}

// ------------------------------------------------------------------------------------------------
// MHA (one query head per KV head).  A tile is 64 tokens = two cache blocks; the query's three bfloat16 terms
// sit in rows 4g..4g+2 of the A operand used for token group g, so after the 16 products lane l holds the
// three partial dot products of token l: one token per lane for the softmax.
// ------------------------------------------------------------------------------------------------
template <int NG>
struct MhaTile {
  u32x4 kc[2], vc[2];
  uint32_t km[NG], vm[NG];
  uint32_t fm;  // fine-half mask word of this lane's 32-row block (only loaded by the PAIRS instantiations)
};

// PAIRS: the cache holds 4-bit tokens as (coarse, fine) pairs of 2-bit rows on (even, odd) rows, flagged in
// a.fine_mask: the two rows' scores add up to the token's score, the token enters the softmax sum once, and each row
// takes the token's weight times its own scale in the value product.
template <int G, bool PAIRS>
__device__ __forceinline__ void decode_mha_body(const DecodeArgs &a) {
  constexpr int NG = kD / G;
  __shared__ float qf[kD];
  // three signed 7-bit digits of q~[e] / U (U a power of two, |q~|/U < 2^20), as int8, in A-operand order of the
  // 16x16x64 int8 product (see k_digit_pos): the code stream's A operand, 16 bytes per lane
  __shared__ __attribute__((aligned(16))) int8_t q_digit[4][kD];  // row 3 stays zero: operand rows that carry nothing
  __shared__ float q_red[kWaves];
  __shared__ __attribute__((aligned(16))) uint16_t q_plain[4][kD];  // terms of q~[e], natural order; row 3 stays zero
  __shared__ __attribute__((aligned(16))) uint16_t w_lds_all[kWaves][2][NG][2][kTokBlock];
  __shared__ __attribute__((aligned(16))) uint16_t zero16[64];  // 128 zero bytes: operand rows that carry nothing
  __shared__ float mrg_m[kWaves], mrg_l[kWaves];
  __shared__ float mrg_o[kWaves][kD];

  const int tid = threadIdx.x;
  // the wavefront index as a scalar: everything derived from it (tile indices, tile addresses) then lives in scalar
  // registers and the loads take a scalar base plus a per-lane offset
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int split = blockIdx.x;
  const int bh = blockIdx.y;  // Hq == Hkv here
  const int mrow = lane & 15, qd = lane >> 4;
  const ExpandK ex;
  auto &w_lds = w_lds_all[wave];  // [blk][group][term][slot]

  // ---- tile bookkeeping and the first two tiles' loads come first: they do not depend on the query, so their
  // latency overlaps with the query rotation below ----
  const int n_tiles = (a.t_win + kMhaTileRows - 1) / kMhaTileRows;  // rows from t_win on are read from the recent-window rings
  int tile_begin, tile_end;
  decode_split_range(n_tiles, a.n_split, split, tile_begin, tile_end);
  const size_t plane_blocks = (size_t)a.T_cap / kTokBlock;
  // Plane bases and tile indices are uniform over the wavefront (scalar registers); a lane adds a fixed 32-bit offset,
  // so every load of the stream is "scalar base + lane offset" and needs no per-lane address arithmetic.
  const gptr_u32 kc_plane = as_global(a.k_codes) + (size_t)bh * plane_blocks * kBlockWords;
  const gptr_u32 vc_plane = as_global(a.v_codes) + (size_t)bh * plane_blocks * kBlockWords;
  const gptr_u32 km_plane = as_global(a.k_meta) + (size_t)bh * a.T_cap * NG;
  const gptr_u32 vm_plane = as_global(a.v_meta) + (size_t)bh * a.T_cap * NG;
  const uint32_t *fm_base = PAIRS ? a.fine_mask + (size_t)(bh / a.Hkv) * plane_blocks + (lane >> 5) : nullptr;
  const uint32_t lane_code = (uint32_t)lane * 4u, lane_meta = (uint32_t)lane * NG;

  auto load_tile = [&](int tile, MhaTile<NG> &t) {
    if constexpr (PAIRS) t.fm = fm_base[2 * tile];
    gptr_u32 kc_t = kc_plane + (size_t)tile * (2 * kBlockWords), vc_t = vc_plane + (size_t)tile * (2 * kBlockWords);
    gptr_u32 km_t = km_plane + (size_t)tile * (64 * NG), vm_t = vm_plane + (size_t)tile * (64 * NG);
    keep_scalar(kc_t); keep_scalar(vc_t); keep_scalar(km_t); keep_scalar(vm_t);
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2) {
      t.kc[b2] = stream_load_x4(kc_t + b2 * kBlockWords + lane_code);
      t.vc[b2] = stream_load_x4(vc_t + b2 * kBlockWords + lane_code);
    }
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      t.km[g] = stream_load_x1(km_t + lane_meta + g);
      t.vm[g] = stream_load_x1(vm_t + lane_meta + g);
    }
  };

  // Three tile buffers: while tile k is consumed, the loads of tiles k+1 and k+2 are in flight.  Loads are issued
  // unconditionally (the index is clamped to the wavefront's last tile) so that the number of outstanding loads is
  // the same on every path and the waits inside the loop count exactly two tiles of loads.
  // the length of the salient list is asked for now and looked at after the stream (the append of a fused decode
  // step does not change it): the 16-bit rows then cost one memory round trip, not three dependent ones
  // (read through the constant address space: a scalar load, whose wait the compiler puts in front of the first use;
  // as a vector load of a uniform address it would be moved to a scalar register, and waited for, right here)
  const int sal_cnt_early = reinterpret_cast<const __attribute__((address_space(4))) int32_t *>(
      reinterpret_cast<uintptr_t>(a.sal_cnt))[bh];
  const int n_mine = tile_begin + wave < tile_end ? (tile_end - tile_begin - wave + kWaves - 1) / kWaves : 0;
  const int last_tile = tile_begin + wave + kWaves * max(n_mine - 1, 0);
  auto tile_at = [&](int k) { return min(tile_begin + wave + kWaves * k, last_tile); };
  MhaTile<NG> tb[3];
  // Fused decode step: the workgroups of the split that owns the row's tile first write the new row (wavefront 1
  // the K row, wavefront 2 the V row, while wavefront 0 stages the query); the barrier below orders those stores
  // before this workgroup's loads of the tile that holds the row, and no other workgroup reads that tile.  A wavefront
  // whose first two tiles include that tile asks for them after the barrier instead of here.
  const bool appends = a.fused_append != 0 && split == a.append_split;  // uniform over the workgroup
  const bool defer_loads = appends && a.t_win == a.T_len && n_mine > 0 &&
                           (tile_at(0) == n_tiles - 1 || tile_at(1) == n_tiles - 1);
  if (n_mine > 0 && !defer_loads) {
    load_tile(tile_at(0), tb[0]);
    load_tile(tile_at(1), tb[1]);
  }
  if (appends && (wave == 1 || wave == 2)) {
    __shared__ __attribute__((aligned(16))) uint8_t step_codes[2][kD];
    __shared__ __attribute__((aligned(16))) uint16_t step_row[2][kD];
    append_row_wave<G>(a.step, bh, wave - 1, lane, step_codes[wave - 1], step_row[wave - 1]);
  }

  if (tid < 64) zero16[tid] = 0;
  if (tid < kD) { q_digit[3][tid] = 0; q_plain[3][tid] = 0; }
  if (wave == 0) rotate_query_lds(a.q + (size_t)bh * kD, qf, a.q_rotated != 0,
                                  a.rope_cos ? a.rope_cos + (size_t)(bh / a.Hkv) * a.rope_stride : nullptr,
                                  a.rope_sin ? a.rope_sin + (size_t)(bh / a.Hkv) * a.rope_stride : nullptr, lane);
  __syncthreads();
  if (defer_loads) {
    load_tile(tile_at(0), tb[0]);
    load_tile(tile_at(1), tb[1]);
  }
  // fixed-point unit of the query: U = 2^ceil(log2 max|q~|) / 2^20 (the digits then cover it exactly, 21 bits)
  float q_unit_inv;
  {
    float mx = tid < kD ? fabsf(qf[tid]) : 0.0f;
    mx = wave_max_dpp(mx);
    if (lane == 0) q_red[wave] = mx;
    __syncthreads();
    mx = fmaxf(fmaxf(q_red[0], q_red[1]), fmaxf(q_red[2], q_red[3]));
    const uint32_t e_biased = min(max(__float_as_uint(mx) >> 23, 20u), 250u);  // mx < 2^(e_biased - 126)
    q_unit_inv = __uint_as_float((273u - e_biased) << 23);                     // 2^20 / 2^(e_biased - 126)
  }
  const float q_unit = 1.0f / q_unit_inv;
  if (tid < kD) {
    const int e = tid;
    const float v = qf[e];
    uint32_t hi, mid, lo;
    split3_bf16(v, hi, mid, lo);
    q_plain[0][e] = (uint16_t)hi; q_plain[1][e] = (uint16_t)mid; q_plain[2][e] = (uint16_t)lo;
    const int n = (int)rintf(v * q_unit_inv);                     // |n| <= 2^20
    const int d2 = (n << 25) >> 25, n1 = (n - d2) >> 7;           // balanced base-128 digits, each in [-64, 64]
    const int d1 = (n1 << 25) >> 25, d0 = (n1 - d1) >> 7;
    const int p = k_digit_pos(e);
    q_digit[0][p] = (int8_t)d0; q_digit[1][p] = (int8_t)d1; q_digit[2][p] = (int8_t)d2;
    qf[e] = (float)n;                                             // the value the digits represent, in units of U
  }
  __syncthreads();

  // ---- per-group sums of the (digitised) query, in units of U ----
  float qsum[NG];
  {
    float qsum_part[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) qsum_part[g] = 0.0f;
#pragma unroll
    for (int rep = 0; rep < 2; ++rep) qsum_part[(NG == 2) ? rep : 0] += qf[lane + 64 * rep];
#pragma unroll
    for (int g = 0; g < NG; ++g) qsum[g] = wave_sum_dpp(qsum_part[g]);
  }

  // ---- A operands for the code stream, per token group g: row 4g+digit carries that digit, other rows are zero.
  // They stay in LDS (two 128-bit reads per product) instead of 32 registers: the kernel then fits three
  // wavefronts per SIMD instead of two, which is what keeps enough loads in flight.
  uint32_t a_off[4];  // byte offset of this lane's operand row inside q_digit, per token group
#pragma unroll
  for (int g = 0; g < 4; ++g) {
    const int dig = mrow - 4 * g;
    a_off[g] = (uint32_t)(((dig >= 0 && dig < 3) ? dig : 3) * kD + qd * 16);
  }
  const ExpandI8 ex8;

  f32x4 acc_o[8];
#pragma unroll
  for (int nb = 0; nb < 8; ++nb) acc_o[nb] = (f32x4){0.f, 0.f, 0.f, 0.f};
  float m_run = -INFINITY, l_run = 0.0f;  // softmax reference (base-2 domain) and this lane's share of the sum
  float swx[NG], szx[NG];                // running sums of w*cx and w*cx*zero over this lane's tokens
#pragma unroll
  for (int g = 0; g < NG; ++g) swx[g] = szx[g] = 0.0f;
  const float sm2 = a.sm_scale * kLog2e;

  const int r16 = lane & 15, half = (lane >> 4) & 1, blk_of_lane = lane >> 5;
  const int slot = 2 * r16 + half, ii = r16 & 3;
  const float cx = pow4_neg(pair_exp(ii)), rcx = 1.0f / cx;  // exact powers of two

  // online-softmax bookkeeping shared by the code stream and the bfloat16 rows.  The reference m_run is only
  // raised when some score exceeds it by more than kLazyMax, so the common tile costs one compare and one branch;
  // weights are then at most 2^kLazyMax, which fp32 sums and the bfloat16 term split absorb.
  auto softmax_step = [&](float score, bool ok, bool count, float &p) -> bool {
    const float sc = ok ? score : -INFINITY;
    if (__ballot(sc > m_run + kLazyMax) != 0ull) {
      const float m_new = wave_max_dpp(sc);
      const float alpha = (m_run == -INFINITY) ? 0.0f : fast_exp2(m_run - m_new);
#pragma unroll
      for (int nb = 0; nb < 8; ++nb) acc_o[nb] *= alpha;
      l_run *= alpha;
#pragma unroll
      for (int g = 0; g < NG; ++g) { swx[g] *= alpha; szx[g] *= alpha; }
      m_run = m_new;
    }
    if (m_run == -INFINITY) { p = 0.0f; return false; }
    p = fast_exp2(sc - m_run);
    l_run += count ? p : 0.0f;  // the fine half of a 4-bit token carries the token's weight but is not a token
    return true;
  };

  // ================= code stream =================
  auto process = [&](const MhaTile<NG> &cur, int tile) {
    const int t = tile * 64 + lane;

    // scores: lane l ends up with the three digit products of token l in acc[0..2] (exact integers)
    i32x4 acc[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) acc[g] = (i32x4){0, 0, 0, 0};
#pragma unroll
    for (int b2 = 0; b2 < 2; ++b2)
#pragma unroll
      for (int hf = 0; hf < 2; ++hf) {
        const int tg = 2 * b2 + hf;
        uint32_t off = a_off[tg];
        asm volatile("" : "+v"(off));  // keep the operand reads inside the loop (see above)
        const i32x4 a0 = *reinterpret_cast<const i32x4 *>(&q_digit[0][0] + off);
        const i32x4 a1 = *reinterpret_cast<const i32x4 *>(&q_digit[0][0] + off + 64);
        acc[0] = mfma_i8(a0, ex8(cur.kc[b2][2 * hf]), acc[0]);
        acc[NG - 1] = mfma_i8(a1, ex8(cur.kc[b2][2 * hf + 1]), acc[NG - 1]);
      }
    float score = 0.0f;
    bool salient = false;
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      const Meta mk = unpack_meta(cur.km[g]);
      salient = salient || mk.salient;
      const float raw = (float)acc[g][0] * 16384.0f + ((float)acc[g][1] * 128.0f + (float)acc[g][2]);
      score += mk.scale * (raw - mk.zero * qsum[g]);
    }
    score *= q_unit;
    score *= sm2;
    const bool ok = (t < a.t_win) && !salient;
    bool count = true;
    if constexpr (PAIRS) {
      const uint32_t from_me = cur.fm >> (lane & 31);      // bit 0: this row is a fine half; bit 1: the next row is
      const bool fine = (from_me & 1u) != 0u, coarse = (from_me & 2u) != 0u;  // pairs start on even rows
      const float partner = dpp_f<0xB1>(score);            // lane ^ 1
      score = (fine || coarse) ? score + partner : score;
      count = !fine;
    }
    float p;
    if (softmax_step(score, ok, count, p)) {
      // weights for the value contraction: w = p * scale_V as two bfloat16 terms, pre-divided by the 4^k of its slot
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        const Meta mv = unpack_meta(cur.vm[g]);
        float hix, lox;
        split2(ok ? p * (mv.scale * cx) : 0.0f, hix, lox);  // rows past T_len hold arbitrary meta
        w_lds[blk_of_lane][g][0][slot] = (uint16_t)hi16(hix);
        w_lds[blk_of_lane][g][1][slot] = (uint16_t)hi16(lox);
        const float wxr = hix + lox;
        swx[g] += wxr;
        szx[g] = __builtin_fmaf(wxr, mv.zero, szx[g]);
      }
      wave_lds_sync();
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2) {
        bf16x8 a_v[NG];
#pragma unroll
        for (int g = 0; g < NG; ++g) {
          const uint16_t *src = mrow < 2 ? &w_lds[b2][g][mrow][8 * qd] : zero16;
          a_v[g] = *reinterpret_cast<const bf16x8 *>(src);
        }
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const int g = (NG == 2) ? (w & 1) : 0;
          const int nbx = 4 * (w & 1) + (w >> 1), nby = nbx + 2;
          acc_o[nbx] = mfma_bf16(a_v[g], ex.x(cur.vc[b2][w]), acc_o[nbx]);
          acc_o[nby] = mfma_bf16(a_v[g], ex.y(cur.vc[b2][w]), acc_o[nby]);
        }
      }
      wave_lds_sync();
    }
  };
  if (n_mine > 0) {
#pragma unroll
    for (int i = 0; i < 2; ++i) {
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2) { settle(tb[i].kc[b2]); settle(tb[i].vc[b2]); }
#pragma unroll
      for (int g = 0; g < NG; ++g) { settle(tb[i].km[g]); settle(tb[i].vm[g]); }
    }
    for (int k = 0; k < n_mine; k += 3) {
      load_tile(tile_at(k + 2), tb[2]);
      process(tb[0], tile_at(k));
      if (k + 1 >= n_mine) break;
      load_tile(tile_at(k + 3), tb[0]);
      process(tb[1], tile_at(k + 1));
      if (k + 2 >= n_mine) break;
      load_tile(tile_at(k + 4), tb[1]);
      process(tb[2], tile_at(k + 2));
    }
  }

  // ================= bfloat16 rows: units of 64 slots dealt to splits, then to wavefronts =========
  // Used twice: the salient overlay (slot = rank in the salient list) and the recent-window rings (slot = row mod W).
  auto bf16_units = [&](const uint16_t *ks_base, const uint16_t *vs_base, int cnt, auto &&row_ok) {
    const int n_units = (cnt + 63) / 64;
    // fused decode step: the 16-bit rows (one of which may be the new row) are read by the appending split only
    const int unit_step = a.fused_append ? kWaves : kWaves * a.n_split;
    const int unit_first = a.fused_append ? (appends ? wave : n_units) : split + wave * a.n_split;
    for (int unit = unit_first; unit < n_units; unit += unit_step) {
      const int s_lane = unit * 64 + lane;
      // only the token groups (16 slots) and blocks (32 slots) that hold rows are touched; the first block of value
      // rows and the row's validity are requested together with the key rows so that the phase costs one round trip
      const int n_grp = min(4, (cnt - unit * 64 + 15) >> 4), n_blk = min(2, (cnt - unit * 64 + 31) >> 5);
      const bool row_valid = row_ok(s_lane);  // fetched whatever cnt says (clamped address): no load behind a branch
      const bool lane_ok = (s_lane < cnt) & row_valid;
      u32x4 vb0[8];
#pragma unroll
      for (int nb = 0; nb < 8; ++nb)
        vb0[nb] = *reinterpret_cast<const u32x4 *>(vs_base + (size_t)(unit * 2) * 4096 + nb * 512 + (16 * qd + mrow) * 8);
      f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll 1
      for (int g = 0; g < n_grp; ++g) {  // one token group at a time keeps the register footprint of this phase small
        const int term = mrow - 4 * g;
        const uint16_t *ap = &q_plain[(term >= 0 && term < 3) ? term : 3][8 * qd];
#pragma unroll
        for (int kc = 0; kc < 4; ++kc) {
          const bf16x8 kb = *reinterpret_cast<const bf16x8 *>(
              ks_base + (size_t)(unit * 64 + 16 * g + mrow) * kD + 32 * kc + 8 * qd);
          acc = mfma_bf16(*reinterpret_cast<const bf16x8 *>(ap + 32 * kc), kb, acc);
        }
      }
      const float score = sm2 * (acc[0] + acc[1] + acc[2]);
      const bool ok = lane_ok;
      float p;
      if (!softmax_step(score, ok, true, p)) continue;
      {
        float hif, lof;
        split2(ok ? p : 0.0f, hif, lof);
        w_lds[blk_of_lane][0][0][slot] = (uint16_t)hi16(hif);
        w_lds[blk_of_lane][0][1][slot] = (uint16_t)hi16(lof);
      }
      wave_lds_sync();
#pragma unroll
      for (int b2 = 0; b2 < 2; ++b2) {
        if (b2 >= n_blk) break;
        const uint16_t *src = mrow < 2 ? &w_lds[b2][0][mrow][8 * qd] : zero16;
        const bf16x8 a_v = *reinterpret_cast<const bf16x8 *>(src);
        // which of this lane's 8 K-slots (pair i, half) are real rows: mask the others (unwritten memory)
        uint32_t keep[4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
          const int s0 = unit * 64 + 32 * b2 + 4 * qd + i;  // half 0; half 1 is 16 slots further
          keep[i] = (s0 < cnt ? 0x0000FFFFu : 0u) | (s0 + 16 < cnt ? 0xFFFF0000u : 0u);
        }
#pragma unroll
        for (int nb = 0; nb < 8; ++nb) {
          u32x4 vb = vb0[nb];
          if (b2 == 1)
            vb = *reinterpret_cast<const u32x4 *>(vs_base + (size_t)(unit * 2 + 1) * 4096 + nb * 512 + (16 * qd + mrow) * 8);
#pragma unroll
          for (int i = 0; i < 4; ++i) vb[i] &= keep[i];
          acc_o[nb] = mfma_bf16(a_v, __builtin_bit_cast(bf16x8, vb), acc_o[nb]);
        }
      }
      wave_lds_sync();
    }
  };
  {
    const int cnt = min(max(sal_cnt_early, 0), a.S_cap);
    const int32_t *sidx = a.sal_idx + (size_t)bh * a.S_cap;
    bf16_units(a.k_sal + (size_t)bh * a.S_cap * kD, a.v_sal + (size_t)bh * a.S_cap * kD, cnt,
               [&](int s) { return sidx[min(s, a.S_cap - 1)] < a.t_win; });  // rows in the window are read there
  }
  if (a.win_len > 0) {
    // slot s holds the row of [t_win, T_len) congruent to s mod W; fine halves and padding rows carry no token
    const int W = a.win_len;
    bf16_units(a.k_win + (size_t)bh * W * kD, a.v_win + (size_t)bh * W * kD, W, [&](int s) {
      int d = (a.T_len - 1 - s) % W;
      d = d < 0 ? d + W : d;
      const int t = a.T_len - 1 - d;
      bool row = t >= a.t_win;
      if constexpr (PAIRS) {
        const int tc = max(t, 0);
        const bool fine = ((a.fine_mask[(size_t)(bh / a.Hkv) * plane_blocks + tc / 32] >> (tc % 32)) & 1u) != 0u;
        const bool pad = (a.k_meta[((size_t)bh * a.T_cap + tc) * NG] & 0xFFFFu) == 0x8000u;
        row = row && !fine && !pad;
      }
      return row;
    });
  }

  // ================= merge the four wavefronts, then either finish (one split) or store the partial =================
  {
    const float l_tot = wave_sum_dpp(l_run);
    float corr[NG];  // what the expansion constant and the zero-points added to every channel of the group
#pragma unroll
    for (int g = 0; g < NG; ++g) corr[g] = kCodeBias * wave_sum_dpp(swx[g]) + wave_sum_dpp(szx[g] * rcx);
    if (lane == 0) { mrg_m[wave] = m_run; mrg_l[wave] = l_tot; }
    if (lane < 16) {
#pragma unroll
      for (int nb = 0; nb < 8; ++nb) {
        mrg_o[wave][16 * nb + lane] = (acc_o[nb][0] + acc_o[nb][1]) - corr[(NG == 2) ? (nb >> 2) : 0];
      }
    }
  }
  __syncthreads();
  float m_all = -INFINITY, l_all = 0.0f, o = 0.0f;
  if (tid < kD) {
#pragma unroll
    for (int w = 0; w < kWaves; ++w) m_all = fmaxf(m_all, mrg_m[w]);
#pragma unroll
    for (int w = 0; w < kWaves; ++w) {
      if (mrg_m[w] == -INFINITY) continue;
      const float wgt = fast_exp2(mrg_m[w] - m_all);
      l_all += wgt * mrg_l[w];
      o += wgt * mrg_o[w][tid];
    }
  }
  if (a.n_split == 1) {
    if (tid < kD) qf[tid] = o / l_all;  // the query is no longer needed: its buffer carries the row to wavefront 0
    if (a.lse && tid == 0) a.lse[bh] = (m_all + __log2f(l_all)) * kLn2;
    __syncthreads();
    if (wave == 0) unrotate_store_wave(qf, a.out, (size_t)bh, a.out_rotated != 0, a.out_half != 0, lane);
  } else if (tid < kD) {
    float *dst = a.partial + ((size_t)bh * a.n_split + split) * kPartialStride;
    if (tid == 0) { dst[0] = m_all; dst[1] = l_all; }
    dst[4 + tid] = o;
  }
}

__global__ __launch_bounds__(64 * kWaves) void decode_mha_kernel_g128(DecodeArgs a) { decode_mha_body<128, false>(a); }
__global__ __launch_bounds__(64 * kWaves) void decode_mha_kernel_g64(DecodeArgs a) { decode_mha_body<64, false>(a); }
__global__ __launch_bounds__(64 * kWaves) void decode_mha_pairs_kernel_g128(DecodeArgs a) {
  decode_mha_body<128, true>(a);
}
__global__ __launch_bounds__(64 * kWaves) void decode_mha_pairs_kernel_g64(DecodeArgs a) {
  decode_mha_body<64, true>(a);
}

// ------------------------------------------------------------------------------------------------
// GQA (R = Hq/Hkv query heads share a KV head, 2 <= R <= 8; also valid for R = 1).  A tile is one cache block
// (32 tokens, two token groups of 16).  Rows 2h+term of the A operand carry the two bfloat16 terms of head h,
// so lane (n, q) receives heads 2q, 2q+1 of token n, and the same lanes own those heads' output rows.
// ------------------------------------------------------------------------------------------------
template <int NG>
struct GqaTile {
  u32x4 kc, vc;
  uint32_t km[2][NG], vm[2][NG];
  uint32_t fm;  // fine-half mask word of the block (only loaded by the PAIRS instantiations)
};

template <int G, bool PAIRS>
__global__ __launch_bounds__(64 * kWaves) void decode_gqa_kernel(DecodeArgs a) {
  constexpr int NG = kD / G;
  __shared__ float qf[8][kD];
  __shared__ __attribute__((aligned(16))) uint16_t q_scaled[16][kD];  // row 2h+term, A-operand order
  __shared__ __attribute__((aligned(16))) uint16_t q_plain[16][kD];   // row 2h+term, natural order
  __shared__ __attribute__((aligned(16))) uint16_t w_lds_all[kWaves][NG][16][kTokBlock];  // [group][row][slot]
  __shared__ float mrg_m[kWaves][8], mrg_l[kWaves][8];
  __shared__ float mrg_o[kWaves][8][kD];

  const int tid = threadIdx.x;
  // the wavefront index as a scalar: everything derived from it (tile indices, tile addresses) then lives in scalar
  // registers and the loads take a scalar base plus a per-lane offset
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6), lane = tid & 63;
  const int split = blockIdx.x;
  const int bh = blockIdx.y;  // b * Hkv + hkv
  const int R = a.Hq / a.Hkv;
  const int b = bh / a.Hkv, hkv = bh % a.Hkv;
  const int mrow = lane & 15, qd = lane >> 4;
  const ExpandK ex;
  auto &w_lds = w_lds_all[wave];

  for (int x = tid; x < 16 * kD; x += 64 * kWaves) { (&q_scaled[0][0])[x] = 0; (&q_plain[0][0])[x] = 0; }
  for (int x = lane; x < NG * 16 * kTokBlock; x += 64) (&w_lds[0][0][0])[x] = 0;
  // Fused decode step: the workgroups of the split that owns the row's tile first write the new row (wavefront 3 the
  // K row, wavefront 2 the V row); the barrier below orders those stores before this workgroup's loads, which all
  // come later, and no other workgroup reads that tile.
  const bool appends = a.fused_append != 0 && split == a.append_split;  // uniform over the workgroup
  if (appends && wave >= 2) {
    __shared__ __attribute__((aligned(16))) uint8_t step_codes[2][kD];
    __shared__ __attribute__((aligned(16))) uint16_t step_row[2][kD];
    append_row_wave<G>(a.step, bh, 3 - wave, lane, step_codes[3 - wave], step_row[3 - wave]);
  }
  for (int h = wave; h < R; h += kWaves) rotate_query_lds(a.q + ((size_t)b * a.Hq + hkv * R + h) * kD, qf[h], a.q_rotated != 0,
                     a.rope_cos ? a.rope_cos + (size_t)b * a.rope_stride : nullptr,
                     a.rope_sin ? a.rope_sin + (size_t)b * a.rope_stride : nullptr, lane);
  __syncthreads();
  // sm_scale * log2(e) is folded into the staged queries (and through them into the bias and group sums), so the
  // products already are base-2 logits
  const float sm2 = a.sm_scale * kLog2e;
  for (int x = tid; x < R * kD; x += 64 * kWaves) {
    const int h = x >> 7, e = x & 127;
    const float v = qf[h][e] * sm2;
    float hif, lof;
    split2(v, hif, lof);
    q_plain[2 * h][e] = (uint16_t)hi16(hif); q_plain[2 * h + 1][e] = (uint16_t)hi16(lof);
    split2(v * pow4_neg(k_channel_exp(e)), hif, lof);
    const int p = k_operand_pos(e);
    q_scaled[2 * h][p] = (uint16_t)hi16(hif); q_scaled[2 * h + 1][p] = (uint16_t)hi16(lof);
  }
  __syncthreads();

  // this lane scores heads h0 = 2*qd and h0+1: their bias / group sums
  const int h0 = 2 * qd;
  float qbias[2][NG], qsum[2][NG];
#pragma unroll
  for (int hh = 0; hh < 2; ++hh) {
    const int h = min(h0 + hh, 7);
    float bias_part[NG], qsum_part[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) bias_part[g] = qsum_part[g] = 0.0f;
    // 16 lanes of the row share the work: lane mrow sums channels mrow, mrow+16, ...
#pragma unroll
    for (int c = 0; c < 8; ++c) {
      const int e = mrow + 16 * c;
      const int g = (NG == 2) ? (c >> 2) : 0;
      bias_part[g] += bf16_bits_to_f32(q_scaled[2 * h][e]) + bf16_bits_to_f32(q_scaled[2 * h + 1][e]);
      qsum_part[g] += (h < R) ? qf[h][e] * sm2 : 0.0f;
    }
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      qbias[hh][g] = kCodeBias * row_sum_dpp(bias_part[g]);
      qsum[hh][g] = row_sum_dpp(qsum_part[g]);
    }
  }

  bf16x8 a_k[4];
#pragma unroll
  for (int kc = 0; kc < 4; ++kc)
    a_k[kc] = *reinterpret_cast<const bf16x8 *>(&q_scaled[mrow][(4 * kc + qd) * 8]);
  f32x4 acc_init[NG];  // rows (head h0: hi, lo; head h0+1: hi, lo): the bias enters through the hi rows
#pragma unroll
  for (int g = 0; g < NG; ++g) acc_init[g] = (f32x4){-qbias[0][g], 0.f, -qbias[1][g], 0.f};

  f32x4 acc_o[8];
#pragma unroll
  for (int nb = 0; nb < 8; ++nb) acc_o[nb] = (f32x4){0.f, 0.f, 0.f, 0.f};
  // Softmax reference (base 2) per head, its trigger level, and this lane's share of the sum.  "No score yet" is a large
  // negative finite number instead of -inf: exp2(x - kNoScore) of a masked score (x = -inf) is 0 and the first real
  // score raises the reference, so neither the weights nor the rescale factor need a special case.
  float m_run[2] = {kNoScore, kNoScore}, m_trig[2] = {kNoScore, kNoScore}, l_run[2] = {0.f, 0.f};
  // Per head and group: szx = running sum of w*cx*zero over this lane's tokens; the sum of the weights themselves
  // (what the expansion constant 128 multiplies) comes out of the matrix cores: one extra product per group and tile
  // against an all-ones operand sums exactly the bfloat16 terms the value product uses, over all 32 slots.
  f32x4 acc_one[NG];
#pragma unroll
  for (int g = 0; g < NG; ++g) acc_one[g] = (f32x4){0.f, 0.f, 0.f, 0.f};
  const bf16x8 ones = __builtin_bit_cast(bf16x8, (u32x4){0x3F803F80u, 0x3F803F80u, 0x3F803F80u, 0x3F803F80u});
  float szx[2][NG];
#pragma unroll
  for (int hh = 0; hh < 2; ++hh)
#pragma unroll
    for (int g = 0; g < NG; ++g) szx[hh][g] = 0.0f;

  // The value product wants every weight divided by the 4^k of its token's slot in the code word (k = pair_exp of
  // the token's position, a per-lane constant).  That factor rides in the exponent of the softmax: weights are taken
  // as exp2(score - (reference + 2k)), i.e. already divided; the sums kept per lane (l_run, szx) carry the same factor
  // and are multiplied by 4^k once at the end.
  const int ii = mrow & 3;  // token n = mrow of its group: pair position
  const float two_k = 2.0f * (float)pair_exp(ii);
  const float rcx = 1.0f / pow4_neg(pair_exp(ii));  // 4^k, exact
  float m_off[2] = {kNoScore, kNoScore};             // reference + 2k
  uint32_t minus_lo = 0x0000BF80u, minus_hi = 0xBF800000u;  // bfloat16 pairs (-1, 0) and (0, -1), kept in registers
  asm volatile("" : "+v"(minus_lo), "+v"(minus_hi));

  // scm[hh][tg]: scores of heads h0+hh for tokens (16*tg + mrow) of the tile, -inf where the row does not take part;
  // returns the weights p[hh][tg] (divided by 4^k).  The reference of a head is raised (and its accumulators rescaled)
  // only when one of its scores exceeds it by more than kLazyMax; the common tile pays one compare and one branch.
  auto softmax_step = [&](const float (&scm)[2][2], const bool (&count)[2], float (&p)[2][2]) {
    float top[2];
    bool need = false;
#pragma unroll
    for (int hh = 0; hh < 2; ++hh) {
      top[hh] = fmaxf(scm[hh][0], scm[hh][1]);
      need = need || (top[hh] > m_trig[hh]);
    }
    if (__ballot(need) != 0ull) {
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        const float mx = row_max_dpp(top[hh]);  // the 16 lanes of a row share a head
        if (mx > m_trig[hh]) {
          const float alpha = fast_exp2(m_run[hh] - mx);  // 0 while there was no score
#pragma unroll
          for (int nb = 0; nb < 8; ++nb) { acc_o[nb][2 * hh] *= alpha; acc_o[nb][2 * hh + 1] *= alpha; }
          l_run[hh] *= alpha;
#pragma unroll
          for (int g = 0; g < NG; ++g) {
            acc_one[g][2 * hh] *= alpha;
            acc_one[g][2 * hh + 1] *= alpha;
            szx[hh][g] *= alpha;
          }
          m_run[hh] = mx;
          m_trig[hh] = mx + kLazyMax;
          m_off[hh] = mx + two_k;
        }
      }
    }
#pragma unroll
    for (int hh = 0; hh < 2; ++hh)
#pragma unroll
      for (int tg = 0; tg < 2; ++tg) {
        p[hh][tg] = fast_exp2(scm[hh][tg] - m_off[hh]);
        l_run[hh] += count[tg] ? p[hh][tg] : 0.0f;  // a fine half carries its token's weight but is not a token
      }
  };
  // upper halves of two floats packed into one word (two bfloat16 values that are already exact in 16 bits)
  auto pack_hi = [](float lo, float hi) {
    return __builtin_amdgcn_perm(__float_as_uint(hi), __float_as_uint(lo), 0x07060302u);
  };

  // ================= code stream =================
  const int n_tiles = (a.t_win + kGqaTileRows - 1) / kGqaTileRows;  // rows from t_win on are read from the recent-window rings
  int tile_begin, tile_end;
  decode_split_range(n_tiles, a.n_split, split, tile_begin, tile_end);
  const size_t plane_blocks = (size_t)a.T_cap / kTokBlock;
  // plane bases and tile indices are uniform (scalar registers); a lane adds a fixed 32-bit offset (see the MHA kernel)
  const gptr_u32 kc_plane = as_global(a.k_codes) + (size_t)bh * plane_blocks * kBlockWords;
  const gptr_u32 vc_plane = as_global(a.v_codes) + (size_t)bh * plane_blocks * kBlockWords;
  const gptr_u32 km_plane = as_global(a.k_meta) + (size_t)bh * a.T_cap * NG;
  const gptr_u32 vm_plane = as_global(a.v_meta) + (size_t)bh * a.T_cap * NG;
  const uint32_t lane_code = (uint32_t)lane * 4u, lane_meta = (uint32_t)mrow * NG;

  const uint32_t *fm_base = PAIRS ? a.fine_mask + (size_t)b * plane_blocks : nullptr;
  auto load_tile = [&](int tile, GqaTile<NG> &t) {
    if constexpr (PAIRS) t.fm = fm_base[tile];
    gptr_u32 kc_t = kc_plane + (size_t)tile * kBlockWords, vc_t = vc_plane + (size_t)tile * kBlockWords;
    gptr_u32 km_t = km_plane + (size_t)tile * (32 * NG), vm_t = vm_plane + (size_t)tile * (32 * NG);
    keep_scalar(kc_t); keep_scalar(vc_t); keep_scalar(km_t); keep_scalar(vm_t);
    t.kc = stream_load_x4(kc_t + lane_code);
    t.vc = stream_load_x4(vc_t + lane_code);
#pragma unroll
    for (int tg = 0; tg < 2; ++tg) {
      if constexpr (NG == 2) {
        const u32x2 k2 = stream_load_x2(km_t + 16 * tg * NG + lane_meta);
        const u32x2 v2 = stream_load_x2(vm_t + 16 * tg * NG + lane_meta);
        t.km[tg][0] = k2[0]; t.km[tg][1] = k2[1];
        t.vm[tg][0] = v2[0]; t.vm[tg][1] = v2[1];
      } else {
        t.km[tg][0] = stream_load_x1(km_t + 16 * tg * NG + lane_meta);
        t.vm[tg][0] = stream_load_x1(vm_t + 16 * tg * NG + lane_meta);
      }
    }
  };

  // Only the last tile of the stream can hold rows at or beyond t_win, whose meta words are arbitrary bits.  For that
  // tile the words of such rows are replaced, in registers, by "salient, scale 0" (K) and "scale 0" (V); everything
  // below then needs no validity mask at all: a salient row gets a score of -inf, hence a weight of exactly 0, and the
  // scales of written rows are finite.
  auto process = [&](const GqaTile<NG> &cur, int tile) {
    uint32_t km[2][NG], vm[2][NG];
#pragma unroll
    for (int tg = 0; tg < 2; ++tg)
#pragma unroll
      for (int g = 0; g < NG; ++g) { km[tg][g] = cur.km[tg][g]; vm[tg][g] = cur.vm[tg][g]; }
    if (tile == n_tiles - 1) {  // uniform over the wavefront
#pragma unroll
      for (int tg = 0; tg < 2; ++tg) {
        const bool beyond = tile * 32 + 16 * tg + mrow >= a.t_win;
#pragma unroll
        for (int g = 0; g < NG; ++g) { km[tg][g] = beyond ? 0x8000u : km[tg][g]; vm[tg][g] = beyond ? 0u : vm[tg][g]; }
      }
    }
    float scm[2][2];
    bool ok[2];
#pragma unroll
    for (int tg = 0; tg < 2; ++tg) {
      f32x4 acc[NG];
#pragma unroll
      for (int g = 0; g < NG; ++g) acc[g] = acc_init[g];  // starts at -128*sum(q'): the expansion constant's share
      const uint32_t w0 = cur.kc[2 * tg], w1 = cur.kc[2 * tg + 1];
      acc[0] = mfma_bf16(a_k[0], ex.x(w0), acc[0]);
      acc[0] = mfma_bf16(a_k[1], ex.y(w0), acc[0]);
      acc[NG - 1] = mfma_bf16(a_k[2], ex.x(w1), acc[NG - 1]);
      acc[NG - 1] = mfma_bf16(a_k[3], ex.y(w1), acc[NG - 1]);
      // bit 15 of every meta word of a salient row is set: as a binary16 pattern the low half is then negative
      const bool off = meta_is_salient(km[tg][0]);
      ok[tg] = !off;
      const float pen = (PAIRS || !off) ? 0.0f : -INFINITY;
      float s0 = pen, s1 = pen;
#pragma unroll
      for (int g = 0; g < NG; ++g) {
        const Meta mk = unpack_meta(km[tg][g]);
        // scale * (dot - 128*sum(q') - zero*sum(q)); the accumulators started at -128*sum(q')
        s0 = __builtin_fmaf(mk.scale, __builtin_fmaf(-mk.zero, qsum[0][g], acc[g][0] + acc[g][1]), s0);
        s1 = __builtin_fmaf(mk.scale, __builtin_fmaf(-mk.zero, qsum[1][g], acc[g][2] + acc[g][3]), s1);
      }
      scm[0][tg] = s0;
      scm[1][tg] = s1;
    }
    bool count[2] = {true, true};
    if constexpr (PAIRS) {
#pragma unroll
      for (int tg = 0; tg < 2; ++tg) {
        const uint32_t from_me = cur.fm >> (16 * tg + mrow);  // bit 0: this row is a fine half; bit 1: the next one is
        const bool pair = (from_me & 3u) != 0u;               // pairs start on even rows: the partner is lane ^ 1
#pragma unroll
        for (int hh = 0; hh < 2; ++hh) {
          const float partner = dpp_f<0xB1>(scm[hh][tg]);
          const float both = pair ? scm[hh][tg] + partner : scm[hh][tg];
          scm[hh][tg] = ok[tg] ? both : -INFINITY;
        }
        count[tg] = (from_me & 1u) == 0u;
      }
    }
    float p[2][2];
    softmax_step(scm, count, p);
    // weights: rows 4*qd + {0,1,2,3} = (head h0: hi, lo; head h0+1: hi, lo); slots 2*mrow (+1 for the second group)
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      float sv[2], zv[2];
#pragma unroll
      for (int tg = 0; tg < 2; ++tg) {
        const Meta mv = unpack_meta(vm[tg][g]);
        sv[tg] = mv.scale;
        zv[tg] = mv.zero;
      }
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        // two bfloat16 terms per weight: hi = the weight rounded to bfloat16, lo = the (exactly representable)
        // remainder rounded to bfloat16; the zero-point sum takes the fp32 weight (it differs from hi+lo by 2^-17
        // relative, on a term of the size of the result itself)
        const float w0 = p[hh][0] * sv[0], w1 = p[hh][1] * sv[1];
        szx[hh][g] = __builtin_fmaf(w0, zv[0], szx[hh][g]);
        szx[hh][g] = __builtin_fmaf(w1, zv[1], szx[hh][g]);
        const uint32_t hi = pack_bf16x2(w0, w1);
        const uint32_t lo = pack_bf16x2(minus_bf16(hi, minus_lo, w0), minus_bf16(hi, minus_hi, w1));
        const int row = 4 * qd + 2 * hh;
        reinterpret_cast<uint32_t *>(&w_lds[g][row][0])[mrow] = hi;
        reinterpret_cast<uint32_t *>(&w_lds[g][row + 1][0])[mrow] = lo;
      }
    }
    wave_lds_sync();
    bf16x8 a_v[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      a_v[g] = *reinterpret_cast<const bf16x8 *>(&w_lds[g][mrow][8 * qd]);
      acc_one[g] = mfma_bf16(a_v[g], ones, acc_one[g]);
    }
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const int g = (NG == 2) ? (w & 1) : 0;
      const int nbx = 4 * (w & 1) + (w >> 1), nby = nbx + 2;
      acc_o[nbx] = mfma_bf16(a_v[g], ex.x(cur.vc[w]), acc_o[nbx]);
      acc_o[nby] = mfma_bf16(a_v[g], ex.y(cur.vc[w]), acc_o[nby]);
    }
    wave_lds_sync();
  };
  // three tile buffers, two tiles of loads in flight (see the MHA kernel)
  // the length of the salient list is asked for now and looked at after the stream (the append of a fused decode
  // step does not change it): the 16-bit rows then cost one memory round trip, not three dependent ones
  // (read through the constant address space: a scalar load, whose wait the compiler puts in front of the first use;
  // as a vector load of a uniform address it would be moved to a scalar register, and waited for, right here)
  const int sal_cnt_early = reinterpret_cast<const __attribute__((address_space(4))) int32_t *>(
      reinterpret_cast<uintptr_t>(a.sal_cnt))[bh];
  const int n_mine = tile_begin + wave < tile_end ? (tile_end - tile_begin - wave + kWaves - 1) / kWaves : 0;
  const int last_tile = tile_begin + wave + kWaves * max(n_mine - 1, 0);
  auto tile_at = [&](int k) { return min(tile_begin + wave + kWaves * k, last_tile); };
  GqaTile<NG> tb[3];
  if (n_mine > 0) {
    load_tile(tile_at(0), tb[0]);
    load_tile(tile_at(1), tb[1]);
#pragma unroll
    for (int i = 0; i < 2; ++i) {
      settle(tb[i].kc); settle(tb[i].vc);
#pragma unroll
      for (int tg = 0; tg < 2; ++tg)
#pragma unroll
        for (int g = 0; g < NG; ++g) { settle(tb[i].km[tg][g]); settle(tb[i].vm[tg][g]); }
    }
    for (int k = 0; k < n_mine; k += 3) {
      load_tile(tile_at(k + 2), tb[2]);
      process(tb[0], tile_at(k));
      if (k + 1 >= n_mine) break;
      load_tile(tile_at(k + 3), tb[0]);
      process(tb[1], tile_at(k + 1));
      if (k + 2 >= n_mine) break;
      load_tile(tile_at(k + 4), tb[1]);
      process(tb[2], tile_at(k + 2));
    }
  }

  // ================= bfloat16 rows: units of 32 slots =================
  // Used twice: the salient overlay (slot = rank in the salient list) and the recent-window rings (slot = row mod W).
  auto bf16_units = [&](const uint16_t *ks_base, const uint16_t *vs_base, int cnt, auto &&row_ok) {
    const int n_units = (cnt + 31) / 32;
    // fused decode step: the 16-bit rows (one of which may be the new row) are read by the appending split only
    const int unit_step = a.fused_append ? kWaves : kWaves * a.n_split;
    const int first_unit = a.fused_append ? (appends ? wave : n_units) : split + wave * a.n_split;
    if (first_unit >= n_units) return;
    bf16x8 a_s[4];
#pragma unroll
    for (int kc = 0; kc < 4; ++kc)
      a_s[kc] = *reinterpret_cast<const bf16x8 *>(&q_plain[mrow][32 * kc + 8 * qd]);
    for (int unit = first_unit; unit < n_units; unit += unit_step) {
      // the value rows and the rows' validity are requested together with the key rows (one round trip for the
      // phase); a token group (16 slots) without rows is not read
      const int n_grp = min(2, (cnt - unit * 32 + 15) >> 4);
      bool lane_ok[2];
#pragma unroll
      for (int tg = 0; tg < 2; ++tg) {
        const int s_lane = unit * 32 + 16 * tg + mrow;
        const bool row_valid = row_ok(s_lane);  // fetched whatever cnt says (clamped address): no load behind a branch
        lane_ok[tg] = (s_lane < cnt) & row_valid;
      }
      u32x4 vb_all[8];
#pragma unroll
      for (int nb = 0; nb < 8; ++nb)
        vb_all[nb] = *reinterpret_cast<const u32x4 *>(vs_base + (size_t)unit * 4096 + nb * 512 + (16 * qd + mrow) * 8);
      float sc[2][2];
      bool ok[2];
#pragma unroll
      for (int tg = 0; tg < 2; ++tg) {
        f32x4 acc = (f32x4){0.f, 0.f, 0.f, 0.f};
        const int s_lane = unit * 32 + 16 * tg + mrow;
        if (tg < n_grp) {
#pragma unroll
          for (int kc = 0; kc < 4; ++kc) {
            const bf16x8 kb =
                *reinterpret_cast<const bf16x8 *>(ks_base + (size_t)s_lane * kD + 32 * kc + 8 * qd);
            acc = mfma_bf16(a_s[kc], kb, acc);
          }
        }
        ok[tg] = lane_ok[tg];
        sc[0][tg] = ok[tg] ? acc[0] + acc[1] : -INFINITY;
        sc[1][tg] = ok[tg] ? acc[2] + acc[3] : -INFINITY;
      }
      float p[2][2];
      const bool count[2] = {true, true};
      softmax_step(sc, count, p);
#pragma unroll
      for (int hh = 0; hh < 2; ++hh) {
        float hif[2], lof[2];
#pragma unroll
        for (int tg = 0; tg < 2; ++tg) split2(p[hh][tg] * rcx, hif[tg], lof[tg]);  // these rows are plain values: undo the 4^-k
        const int row = 4 * qd + 2 * hh;
        reinterpret_cast<uint32_t *>(&w_lds[0][row][0])[mrow] = pack_hi(hif[0], hif[1]);
        reinterpret_cast<uint32_t *>(&w_lds[0][row + 1][0])[mrow] = pack_hi(lof[0], lof[1]);
      }
      wave_lds_sync();
      const bf16x8 a_v = *reinterpret_cast<const bf16x8 *>(&w_lds[0][mrow][8 * qd]);
      uint32_t keep[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) {
        const int s0 = unit * 32 + 4 * qd + i;
        keep[i] = (s0 < cnt ? 0x0000FFFFu : 0u) | (s0 + 16 < cnt ? 0xFFFF0000u : 0u);
      }
#pragma unroll
      for (int nb = 0; nb < 8; ++nb) {
        u32x4 vb = vb_all[nb];
#pragma unroll
        for (int i = 0; i < 4; ++i) vb[i] &= keep[i];
        acc_o[nb] = mfma_bf16(a_v, __builtin_bit_cast(bf16x8, vb), acc_o[nb]);
      }
      wave_lds_sync();
    }
  };
  {
    const int cnt = min(max(sal_cnt_early, 0), a.S_cap);
    const int32_t *sidx = a.sal_idx + (size_t)bh * a.S_cap;
    bf16_units(a.k_sal + (size_t)bh * a.S_cap * kD, a.v_sal + (size_t)bh * a.S_cap * kD, cnt,
               [&](int s) { return sidx[min(s, a.S_cap - 1)] < a.t_win; });  // rows in the window are read there
  }
  if (a.win_len > 0) {
    // slot s holds the row of [t_win, T_len) congruent to s mod W; fine halves and padding rows carry no token
    const int W = a.win_len;
    bf16_units(a.k_win + (size_t)bh * W * kD, a.v_win + (size_t)bh * W * kD, W, [&](int s) {
      int d = (a.T_len - 1 - s) % W;
      d = d < 0 ? d + W : d;
      const int t = a.T_len - 1 - d;
      bool row = t >= a.t_win;
      if constexpr (PAIRS) {
        const int tc = max(t, 0);
        const bool fine = ((a.fine_mask[(size_t)b * plane_blocks + tc / 32] >> (tc % 32)) & 1u) != 0u;
        const bool pad = (a.k_meta[((size_t)bh * a.T_cap + tc) * NG] & 0xFFFFu) == 0x8000u;
        row = row && !fine && !pad;
      }
      return row;
    });
  }

  // ================= merge the four wavefronts =================
#pragma unroll
  for (int hh = 0; hh < 2; ++hh) {
    const int h = h0 + hh;
    const float l_tot = row_sum_dpp(l_run[hh] * rcx);
    float corr[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g)  // acc_one already holds the sum over all slots (every column the same)
      corr[g] = kCodeBias * (acc_one[g][2 * hh] + acc_one[g][2 * hh + 1]) + row_sum_dpp(szx[hh][g] * rcx);
    if (mrow == 0) { mrg_m[wave][h] = m_run[hh]; mrg_l[wave][h] = l_tot; }
#pragma unroll
    for (int nb = 0; nb < 8; ++nb) {
      mrg_o[wave][h][16 * nb + mrow] = (acc_o[nb][2 * hh] + acc_o[nb][2 * hh + 1]) - corr[(NG == 2) ? (nb >> 2) : 0];
    }
  }
  __syncthreads();
  for (int h = 0; h < R; ++h) {
    float m_all = -INFINITY, l_all = 0.0f, o = 0.0f;
    if (tid < kD) {
#pragma unroll
      for (int w = 0; w < kWaves; ++w) m_all = fmaxf(m_all, mrg_m[w][h]);
#pragma unroll
      for (int w = 0; w < kWaves; ++w) {
        const float wgt = fast_exp2(mrg_m[w][h] - m_all);  // a wavefront without scores has kNoScore and sums of 0
        l_all += wgt * mrg_l[w][h];
        o += wgt * mrg_o[w][h][tid];
      }
    }
    const size_t bhq = (size_t)b * a.Hq + hkv * R + h;
    if (a.n_split == 1) {
      if (tid < kD) qf[h][tid] = o / l_all;  // the queries are no longer needed: their buffers carry the rows
      if (a.lse && tid == 0) a.lse[bhq] = (m_all + __log2f(l_all)) * kLn2;
    } else if (tid < kD) {
      float *dst = a.partial + (bhq * a.n_split + split) * kPartialStride;
      if (tid == 0) { dst[0] = m_all; dst[1] = l_all; }
      dst[4 + tid] = o;
    }
  }
  if (a.n_split == 1) {
    __syncthreads();
    for (int h = wave; h < R; h += kWaves)
      unrotate_store_wave(qf[h], a.out, (size_t)b * a.Hq + hkv * R + h, a.out_rotated != 0, a.out_half != 0, lane);
  }
}

// ------------------------------------------------------------------------------------------------
// Merge the KV splits (exact log-sum-exp merge), rotate the output back (H is its own inverse), write out.
// ------------------------------------------------------------------------------------------------
__global__ __launch_bounds__(128) void decode_combine_kernel(DecodeArgs a) {
  __shared__ float of[kD];
  const int bhq = blockIdx.x;
  const int d = threadIdx.x;
  const float *part = a.partial + (size_t)bhq * a.n_split * kPartialStride;
  float m_all = -INFINITY;
  for (int s = 0; s < a.n_split; ++s) m_all = fmaxf(m_all, part[(size_t)s * kPartialStride]);
  float l_all = 0.0f, o = 0.0f;
  for (int s = 0; s < a.n_split; ++s) {
    const float ms = part[(size_t)s * kPartialStride];
    if (ms == -INFINITY) continue;
    const float wgt = fast_exp2(ms - m_all);
    l_all += wgt * part[(size_t)s * kPartialStride + 1];
    o += wgt * part[(size_t)s * kPartialStride + 4 + d];
  }
  of[d] = o / l_all;
  if (a.lse && d == 0) a.lse[bhq] = (m_all + __log2f(l_all)) * kLn2;
  __syncthreads();
  if (d < kWave) unrotate_store_wave(of, a.out, (size_t)bhq, a.out_rotated != 0, a.out_half != 0, d);
}

}  // namespace

hipError_t launch_decode_attention(const DecodeArgs &a_in, int G, hipStream_t stream) {
  DecodeArgs a = a_in;
  {
    const int rows = a.Hq == a.Hkv ? kMhaTileRows : kGqaTileRows;
    a.append_split = decode_last_tile_split((a.t_win + rows - 1) / rows, a.n_split);
  }
  dim3 grid(a.n_split, a.B * a.Hkv), block(64 * kWaves);
  if (a.Hq == a.Hkv) {
    if (a.fine_mask) {
      if (G == 128) hipLaunchKernelGGL(decode_mha_pairs_kernel_g128, grid, block, 0, stream, a);
      else hipLaunchKernelGGL(decode_mha_pairs_kernel_g64, grid, block, 0, stream, a);
    } else {
      if (G == 128) hipLaunchKernelGGL(decode_mha_kernel_g128, grid, block, 0, stream, a);
      else hipLaunchKernelGGL(decode_mha_kernel_g64, grid, block, 0, stream, a);
    }
  } else if (a.fine_mask) {
    if (G == 128) hipLaunchKernelGGL((decode_gqa_kernel<128, true>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((decode_gqa_kernel<64, true>), grid, block, 0, stream, a);
  } else {
    if (G == 128) hipLaunchKernelGGL((decode_gqa_kernel<128, false>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((decode_gqa_kernel<64, false>), grid, block, 0, stream, a);
  }
  hipError_t e = hipGetLastError();
  if (e != hipSuccess || a.n_split == 1) return e;
  hipLaunchKernelGGL(decode_combine_kernel, dim3(a.B * a.Hq), dim3(128), 0, stream, a);
  return hipGetLastError();
}

}  // namespace akvq

// Per-row quantization shared by the write path's kernels and by the fused decode step: Eq. 5-6 for one group, the code
// of Eq. 3, and the single-row append (one wavefront per row and tensor).
#pragma once
#include "akvq_device.h"
#include "akvq_kernels.h"

namespace akvq {
namespace {

// value of a stored 16-bit row before its conversion: u * scale rounded once, with a zero product stored as +0
// (lanes that hold negated butterfly values cannot know the sign of a zero; x * y + (+0) is +0 for either sign)
__device__ __forceinline__ float scaled_row_value(float u, float scale) { return __fmaf_rn(u, scale, 0.0f); }

struct GroupQ {
  uint32_t meta;      // scale bits | zero << 16 (salient flag added by the caller)
  float rcpu;         // kappa / scale
  float magic_zero;   // 1.5 * 2^23 + zero
  uint32_t s16;       // scale bits and zero-point on their own (the 4-bit tier splits them over two rows)
  int z;
};
// number of levels of the two tiers: 1/(2^n - 1) rounded to binary32, and the largest stored scale (the 4-bit tier
// keeps 4*scale representable in binary16)
struct TierQ {
  float inv_levels;
  uint32_t s16_max;
};
__device__ __forceinline__ TierQ tier_two_bit() { return {__uint_as_float(0x3EAAAAABu), 0x7BFFu}; }
__device__ __forceinline__ TierQ tier_four_bit() { return {__uint_as_float(0x3D888889u), 0x73FFu}; }

constexpr float kMagic = 12582912.0f;      // 1.5 * 2^23: adding it rounds to an integer in the low mantissa bits
constexpr uint32_t kMagicBits = 0x4B400000u;

// Eq. 5-6 for one group from the extrema of the un-normalised transform.
__device__ __forceinline__ GroupQ group_params(float umin, float umax, float kappa, float clip, TierQ tq) {
  float gmin = __fmul_rn(umin, kappa), gmax = __fmul_rn(umax, kappa);
  float cmin = __fmul_rn(clip, gmin), cmax = __fmul_rn(clip, gmax);
  float range = __fsub_rn(cmax, cmin);
  float s32 = __fmul_rn(range, tq.inv_levels);
  // smallest binary16 >= s32: one conversion with the 16/64-bit rounding mode switched to "toward +infinity" around
  // it (bits 3:2 of the MODE register; the mode is back to nearest-even before any other instruction runs);
  // +infinity (0x7C00) and anything above the tier's largest scale end at that largest scale
  uint32_t s16;
  asm volatile("s_setreg_imm32_b32 hwreg(HW_REG_MODE, 2, 2), 1\n\t"
               "v_cvt_f16_f32 %0, %1\n\t"
               "s_setreg_imm32_b32 hwreg(HW_REG_MODE, 2, 2), 0"
               : "=v"(s16) : "v"(s32));
  s16 = min(s16 & 0xFFFFu, tq.s16_max);
  if (!(s32 > 0.0f)) s16 = 0x3C00u;
  float s = half_bits_to_float(s16);
  // 1/s correctly rounded: s has an 11-bit significand (binary16), so 1/s is either exact or at least 2^-35 (relative)
  // away from any rounding boundary of fp32, far more than the 2^-45 error left by one Newton step on the hardware
  // reciprocal (accurate to 1 ulp); the fused step rounds once.
  const float r0 = __builtin_amdgcn_rcpf(s);
  float rcp = __builtin_fmaf(r0, __builtin_fmaf(-s, r0, 1.0f), r0);
  float zr = rintf(__fmul_rn(cmin, rcp));
  zr = (zr != zr) ? 0.0f : zr;
  const float zf = __builtin_amdgcn_fmed3f(-zr, -32768.0f, 32767.0f);  // the zero-point, saturated to int16, still a float
  const int z = (int)zf;
  GroupQ g;
  g.meta = s16 | ((uint32_t)z << 16);
  g.rcpu = __fmul_rn(rcp, kappa);
  g.magic_zero = kMagic + zf;  // exact: an integer below 2^22 on top of 1.5 * 2^23
  g.s16 = s16;
  g.z = z;
  return g;
}

// Eq. 3: clamp(round(x/scale + zero), 0, 3); the fused multiply-add rounds the exact sum once, to an integer.
// Returns the bit pattern of 1.5*2^23 + code: the code sits in the two low bits, the rest is the constant kMagicBits.
__device__ __forceinline__ uint32_t code_bits(float u, const GroupQ &g) {
  float t = __fmaf_rn(u, g.rcpu, g.magic_zero);
  t = fminf(fmaxf(t, kMagic), kMagic + 3.0f);
  return __float_as_uint(t);
}
// The same for a row of any tier: clamp to the tier's top level, then extract the field this row stores (bits 2-3 of
// a 4-bit code for the coarse half, bits 0-1 otherwise, nothing for a padding row): one bit-field extract.  Returns the
// bare field (no constant part), so the tiered kernel packs without the bias constants.
__device__ __forceinline__ uint32_t code_bits_tiered(float u, const GroupQ &g, float top, uint32_t shift, uint32_t width) {
  float t = __fmaf_rn(u, g.rcpu, g.magic_zero);
  t = fminf(fmaxf(t, kMagic), top);
  return __builtin_amdgcn_ubfe(__float_as_uint(t), shift, width);
}
// ------------------------------------------------------------------------------------------------
// One new row per (batch, kv-head): the decode step.  The block kernel above spends a whole wavefront, and a few
// thousand instructions fetched once, on a 32-token block that holds a single new token; here one wavefront owns one
// row of one tensor: lane l holds channels l and l + 64, so the stride-64 butterfly (and the rotary pair) is inside
// the lane and the other six strides are lane exchanges.  Same arithmetic as the block kernel: every butterfly is
// (lower + upper, lower - upper) on the same pairs in the same stride order, so the stored bits are identical.
// Codes are gathered through LDS into the words of the packed planes; V words (two codes of this token each, 64
// words) and K words (16 codes each, 8 words) are read, merged and written back.
// ------------------------------------------------------------------------------------------------
__device__ __forceinline__ float xor_butterfly(float v, int s, int lane) {
  const float p = __shfl_xor(v, s, kWave);
  return (lane & s) ? (p - v) : (v + p);
}
__device__ __forceinline__ float wave_min_all(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fminf(v, __shfl_xor(v, off, kWave));
  return v;
}
__device__ __forceinline__ float wave_max_all(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
  return v;
}

// One wavefront writes row a.T_len of (batch, kv-head) bh of one tensor (0 = K, 1 = V); code_lds (128 bytes) and
// row_lds (128 x 16 bit) are scratch of this wavefront alone.
template <int G>
__device__ __forceinline__ void append_row_wave(const QuantArgs &a, int bh, int tensor, int lane, uint8_t *code_lds,
                                                uint16_t *row_lds) {
  constexpr int NG = kD / G;
  const int t = a.T_len;          // the row being written
  const int blk = t / kTokBlock, half = (t % kTokBlock) >> 4, n16 = t & 15;
  const bool rotate = (tensor == 0 ? a.rotate_k : a.rotate_v) != 0;
  const float kappa = rotate ? inv_sqrt128() : 1.0f;

  // everything that has to come from memory is requested first
  const int32_t *sidx = a.sal_idx + (size_t)bh * a.S_cap;
  int cnt = a.sal_cnt[bh];
  const int first_entry = sidx[lane];  // S_cap >= 64: asked for together with the count instead of after it
  const uint16_t *row = (tensor == 0 ? a.k_new : a.v_new) + (size_t)bh * kD;
  float x0 = half_bits_to_float(row[lane]), x1 = half_bits_to_float(row[lane + 64]);
  const size_t blk_word = ((size_t)bh * (a.T_cap / kTokBlock) + blk) * kBlockWords;
  uint32_t *v_word = a.v_codes + blk_word + 64 * (n16 >> 2) + lane;                       // tensor 1: lane's word
  uint32_t *k_word = a.k_codes + blk_word + (size_t)(16 * (lane >> 1) + n16) * 4 + 2 * half + (lane & 1);  // lanes 0..7
  uint32_t old_word = 0u;  // a V word also holds seven other tokens; a K word holds this token only
  if (tensor == 1) old_word = *v_word;
  if (tensor == 0 && a.rope_cos != nullptr) {
    const size_t at = (size_t)(bh / a.Hkv) * a.rope_stride + lane;
    const float c = half_bits_to_float(a.rope_cos[at]), sn = half_bits_to_float(a.rope_sin[at]);
    float r0 = __fmaf_rn(x0, c, -__fmul_rn(x1, sn)), r1 = __fmaf_rn(x1, c, __fmul_rn(x0, sn));
    asm("" : "+v"(r0));  // keeps the rounding to fp32 and the one to binary16 apart
    asm("" : "+v"(r1));
    x0 = half_bits_to_float(float_to_half_bits_rne(r0));
    x1 = half_bits_to_float(float_to_half_bits_rne(r1));
  }

  // is the row listed as salient, and at which rank?
  cnt = min(max(cnt, 0), a.S_cap);
  int slot = -1;
  for (int base = 0; base < cnt; base += kWave) {
    const int e = base + lane < cnt ? (base == 0 ? first_entry : sidx[base + lane]) : -1;
    const unsigned long long hit = __ballot(e == t);
    if (hit != 0ull) slot = base + __builtin_ctzll(hit);
  }

  if (rotate) {
#pragma unroll
    for (int s = 1; s < 64; s <<= 1) {
      x0 = xor_butterfly(x0, s, lane);
      x1 = xor_butterfly(x1, s, lane);
    }
    const float lo = x0 + x1, hi = x0 - x1;
    x0 = lo;
    x1 = hi;
  }

  GroupQ gq[2];
  if constexpr (NG == 1) {
    const float mn = wave_min_all(fminf(x0, x1)), mx = wave_max_all(fmaxf(x0, x1));
    gq[0] = gq[1] = group_params(mn, mx, kappa, a.clip, tier_two_bit());
  } else {
    gq[0] = group_params(wave_min_all(x0), wave_max_all(x0), kappa, a.clip, tier_two_bit());
    gq[1] = group_params(wave_min_all(x1), wave_max_all(x1), kappa, a.clip, tier_two_bit());
  }
  const uint32_t c0 = code_bits(x0, gq[0]) & 3u, c1 = code_bits(x1, gq[1]) & 3u;
  code_lds[lane] = (uint8_t)c0;
  code_lds[lane + 64] = (uint8_t)c1;
  const uint32_t y0 = pack_bf16x2(scaled_row_value(x0, kappa), 0.0f) & 0xFFFFu, y1 = pack_bf16x2(scaled_row_value(x1, kappa), 0.0f) & 0xFFFFu;
  row_lds[lane] = (uint16_t)y0;
  row_lds[lane + 64] = (uint16_t)y1;
  wave_lds_sync();

  if (lane == 0) {
    uint32_t *meta = (tensor == 0 ? a.k_meta : a.v_meta) + ((size_t)bh * a.T_cap + t) * NG;
    meta[0] = gq[0].meta | (slot >= 0 ? 0x8000u : 0u);
    if constexpr (NG == 2) meta[1] = gq[1].meta | (slot >= 0 ? 0x8000u : 0u);
  }

  if (tensor == 0) {
    if (lane < 8) {
      // word (j, mh) = lane (j = lane / 2, mh = lane % 2): slot 8*ml + i holds channel 64*mh + 32*ml + 8*j + i
      const int j = lane >> 1, mh = lane & 1;
      uint32_t word = 0u;
#pragma unroll
      for (int ml = 0; ml < 2; ++ml) {
        const u32x2 eight = *reinterpret_cast<const u32x2 *>(&code_lds[64 * mh + 32 * ml + 8 * j]);
#pragma unroll
        for (int i = 0; i < 8; ++i)
          word |= ((eight[i >> 2] >> (8 * (i & 3))) & 3u) << (2 * (8 * ml + i));
      }
      *k_word = word;  // the word holds this token's codes only
    }
  } else {
    // word lane: n = lane / 4, nb = (lane / 2) % 2 + 2 * XY + 4 * (lane % 2); XY = 0, 1 sit 8 bits apart
    const int n = lane >> 2, nb_lo = ((lane >> 1) & 1) + 4 * (lane & 1);
    const uint32_t cx = code_lds[16 * nb_lo + n], cy = code_lds[16 * (nb_lo + 2) + n];
    const int bit = 16 * half + 2 * (n16 & 3);
    const uint32_t mask = (3u << bit) | (3u << (bit + 8));
    *v_word = (old_word & ~mask) | (cx << bit) | (cy << (bit + 8));
  }

  // 16-bit copies: overlay slot of a salient row, ring slot of the recent window (the new row is always inside it)
  auto store_row16 = [&](uint16_t *k_rows, uint16_t *v_plane, int s16) {
    if (tensor == 0) {
      reinterpret_cast<uint32_t *>(k_rows + (size_t)s16 * kD)[lane] = reinterpret_cast<const uint32_t *>(row_lds)[lane];
    } else {
      const int sb = s16 >> 5, sh = (s16 & 31) >> 4, sr = s16 & 15, sq = sr >> 2, sii = sr & 3;
#pragma unroll
      for (int k = 0; k < 2; ++k) {
        const int e = lane + 64 * k, nb = e >> 4, n = e & 15;
        v_plane[(size_t)sb * 4096 + nb * 512 + (16 * sq + n) * 8 + 2 * sii + sh] = (uint16_t)(k == 0 ? y0 : y1);
      }
    }
  };
  if (slot >= 0) store_row16(a.k_sal + (size_t)bh * a.S_cap * kD, a.v_sal + (size_t)bh * a.S_cap * kD, slot);
  if (a.win_len > 0)
    store_row16(a.k_win + (size_t)bh * a.win_len * kD, a.v_win + (size_t)bh * a.win_len * kD, t % a.win_len);
}

}  // namespace
}  // namespace akvq

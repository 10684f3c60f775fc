// Write path of the AKVQ-VL cache (Section III-C of arXiv 2501.15021): rotate each new Key/Value head vector by
// the 128-point Walsh-Hadamard matrix (Eq. 7), derive per-group scale and zero-point (Eq. 5-6, with clipping),
// emit 2-bit codes (Eq. 3), pack them into the block layout decode reads, and keep salient rows as bfloat16.
//
// Mapping: one wavefront owns one 32-token block of one (batch, kv-head, tensor).  Four neighbouring lanes own a
// token pair (t, t+16): lane (r, j) holds channels e = 32*m + 8*j + i (m<4, i<8) of tokens r and r+16 of the
// block, so every global load is a 128-bit load and a quad covers 64 contiguous bytes of a row.  Butterfly
// strides 1,2,4 and 32,64 stay in registers; strides 8,16 cross the quad with DPP quad_perm.
#include "../../include/akvq.h"
#include "akvq_device.h"
#include "akvq_kernels.h"
#include "akvq_rowquant.h"

namespace akvq {

namespace {

template <int CTRL>
__device__ __forceinline__ uint32_t dpp_move_u(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}
// Running extrema, three operands at a time, and their reduction over the four lanes of a quad with the partner's
// value read through DPP by the min / max itself.  Assembly, because the compiler's fminf / fmaxf first canonicalise
// operands it cannot prove quiet (one more instruction each) and reach a partner lane through a separate move.
__device__ __forceinline__ void minmax3(float &mn, float &mx, float a, float b) {
  asm("v_min3_f32 %0, %0, %1, %2" : "+v"(mn) : "v"(a), "v"(b));
  asm("v_max3_f32 %0, %0, %1, %2" : "+v"(mx) : "v"(a), "v"(b));
}
// (the leading s_nop covers the wait states of a DPP read after a VALU write of its source and after an EXEC write)
__device__ __forceinline__ void quad_minmax(float &mn, float &mx) {
  asm volatile("s_nop 4\n\t"
               "v_min_f32_dpp %0, %0, %0 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
               "v_max_f32_dpp %1, %1, %1 quad_perm:[1,0,3,2] row_mask:0xf bank_mask:0xf\n\t"
               "s_nop 1\n\t"
               "v_min_f32_dpp %0, %0, %0 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf\n\t"
               "v_max_f32_dpp %1, %1, %1 quad_perm:[2,3,0,1] row_mask:0xf bank_mask:0xf"
               : "+v"(mn), "+v"(mx));
}
constexpr int kRowRor4 = 0x124;  // rotate right by 4 inside a row of 16 lanes
constexpr int kRowRor8 = 0x128;

// A cross-lane butterfly level: the lane whose index bit is clear keeps a+b, its partner should keep a-b (a = the
// lower lane's value).  One DPP multiply-add per element does it: own += c * partner with c = +1 in the lower lane and
// -1 in the upper one.  The product is exact and the sum is rounded once, exactly like the add of the specification;
// the upper lane ends up with b-a, i.e. the negated result, and since every later level is linear that lane simply
// carries all its values negated from then on (rounding to nearest is symmetric in sign).  After both cross-lane
// levels lanes j = 1, 2 hold negated values; quad_sign(j) is folded into the per-lane constants that consume them.
__device__ __forceinline__ float quad_sign(int j) { return (j == 1 || j == 2) ? -1.0f : 1.0f; }

// Eight elements of one level.  The leading s_nop covers the wait states a DPP read needs after the VALU write of
// its source register (and after an EXEC write): the compiler does not track hazards of inline assembly.
#define AKVQ_DPP_FMAC8(CTRL, NOP)                                                                              \
  asm volatile("s_nop " NOP "\n\t"                                                                            \
               "v_fmac_f32_dpp %0, %0, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                            \
               "v_fmac_f32_dpp %1, %1, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                            \
               "v_fmac_f32_dpp %2, %2, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                            \
               "v_fmac_f32_dpp %3, %3, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                            \
               "v_fmac_f32_dpp %4, %4, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                            \
               "v_fmac_f32_dpp %5, %5, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                            \
               "v_fmac_f32_dpp %6, %6, %8 " CTRL " row_mask:0xf bank_mask:0xf\n\t"                            \
               "v_fmac_f32_dpp %7, %7, %8 " CTRL " row_mask:0xf bank_mask:0xf"                                \
               : "+v"(x[0]), "+v"(x[1]), "+v"(x[2]), "+v"(x[3]), "+v"(x[4]), "+v"(x[5]), "+v"(x[6]), "+v"(x[7]) \
               : "v"(c))
__device__ __forceinline__ void quad_level_xor1(float (&x)[8], float c, bool first) {
  if (first) AKVQ_DPP_FMAC8("quad_perm:[1,0,3,2]", "4"); else AKVQ_DPP_FMAC8("quad_perm:[1,0,3,2]", "1");
}
__device__ __forceinline__ void quad_level_xor2(float (&x)[8], float c, bool first) {
  if (first) AKVQ_DPP_FMAC8("quad_perm:[2,3,0,1]", "4"); else AKVQ_DPP_FMAC8("quad_perm:[2,3,0,1]", "1");
}
#undef AKVQ_DPP_FMAC8

// First level (stride 1) straight from the packed binary16 pair: lo + hi and lo - hi, each one mixed-precision
// multiply-add (the widening is exact, the sum is rounded once, as widening followed by an fp32 add would be).
__device__ __forceinline__ void level1_from_half2(uint32_t w, float &sum, float &diff) {
  asm("v_fma_mix_f32 %0, %1, 1.0, %1 op_sel:[0,0,1] op_sel_hi:[1,0,1]" : "=v"(sum) : "v"(w));
  asm("v_fma_mix_f32 %0, %1, 1.0, -%1 op_sel:[0,0,1] op_sel_hi:[1,0,1]" : "=v"(diff) : "v"(w));
}

// un-normalised 128-point butterfly of one row held as raw[m] (eight binary16 channels 32m+8j..+7 per m) with the j
// index spread over the quad; the result in lane j is quad_sign(j) times the transform
__device__ __forceinline__ void wht128_quad(const u32x4 (&raw)[4], float (&u)[4][8], int j) {
  // stride 1
#pragma unroll
  for (int m = 0; m < 4; ++m)
#pragma unroll
    for (int w = 0; w < 4; ++w) level1_from_half2(raw[m][w], u[m][2 * w], u[m][2 * w + 1]);
  // strides 2, 4: inside i
#pragma unroll
  for (int h = 2; h < 8; h *= 2)
#pragma unroll
    for (int m = 0; m < 4; ++m)
#pragma unroll
      for (int i = 0; i < 8; ++i)
        if ((i & h) == 0) {
          float a = u[m][i], b = u[m][i + h];
          u[m][i] = a + b;
          u[m][i + h] = a - b;
        }
  // strides 8, 16: across the quad (j bit 0, j bit 1)
  const float c1 = (j & 1) ? -1.0f : 1.0f, c2 = (j & 2) ? -1.0f : 1.0f;
#pragma unroll
  for (int m = 0; m < 4; ++m) quad_level_xor1(u[m], c1, m == 0);
#pragma unroll
  for (int m = 0; m < 4; ++m) quad_level_xor2(u[m], c2, m == 0);
  // strides 32, 64: inside m
#pragma unroll
  for (int h = 1; h < 4; h *= 2)
#pragma unroll
    for (int m = 0; m < 4; ++m)
      if ((m & h) == 0)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          float a = u[m][i], b = u[m + h][i];
          u[m][i] = a + b;
          u[m + h][i] = a - b;
        }
}

// Rotary position embedding of one row held as raw[m] (see wht128_quad): channel e pairs with e + 64, i.e. raw[mm] with
// raw[mm + 2] word by word, both in this lane; cw / sw hold the binary16 cos / sin of channels 32*mm + 8*j .. + 7.
// Both products are exact in fp32 and the multiply-add rounds their sum once; the result is then rounded to binary16.
// The mixed-precision instructions read the binary16 halves in place (HI selects the upper half of every word); being
// assembly, they also keep the compiler from merging the two roundings into one.
template <int HI>
__device__ __forceinline__ float rope_mix(uint32_t x, uint32_t c, uint32_t xp, uint32_t sn, bool subtract) {
  float t, r;
  const float neg_zero = -0.0f;  // product + (-0) is the product itself, signed zeros included
  if (HI) asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,1,0] op_sel_hi:[1,1,0]" : "=v"(t) : "v"(xp), "v"(sn), "v"(neg_zero));
  else asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[1,1,0]" : "=v"(t) : "v"(xp), "v"(sn), "v"(neg_zero));
  if (subtract) {
    if (HI) asm("v_fma_mix_f32 %0, %1, %2, -%3 op_sel:[1,1,0] op_sel_hi:[1,1,0]" : "=v"(r) : "v"(x), "v"(c), "v"(t));
    else asm("v_fma_mix_f32 %0, %1, %2, -%3 op_sel:[0,0,0] op_sel_hi:[1,1,0]" : "=v"(r) : "v"(x), "v"(c), "v"(t));
  } else {
    if (HI) asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,1,0] op_sel_hi:[1,1,0]" : "=v"(r) : "v"(x), "v"(c), "v"(t));
    else asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[1,1,0]" : "=v"(r) : "v"(x), "v"(c), "v"(t));
  }
  return r;
}
__device__ __forceinline__ void rope_row_quad(u32x4 (&raw)[4], const u32x4 (&cw)[2], const u32x4 (&sw)[2]) {
#pragma unroll
  for (int mm = 0; mm < 2; ++mm)
#pragma unroll
    for (int w = 0; w < 4; ++w) {
      const uint32_t lo = raw[mm][w], hi = raw[mm + 2][w], c = cw[mm][w], sn = sw[mm][w];
      raw[mm][w] = float_to_half_bits_rne(rope_mix<0>(lo, c, hi, sn, true)) |
                   (float_to_half_bits_rne(rope_mix<1>(lo, c, hi, sn, true)) << 16);
      raw[mm + 2][w] = float_to_half_bits_rne(rope_mix<0>(hi, c, lo, sn, false)) |
                       (float_to_half_bits_rne(rope_mix<1>(hi, c, lo, sn, false)) << 16);
    }
}

// Packing adds the raw patterns with shifts (one shift-add per code); what the constant part of every pattern
// contributes is a compile-time constant (mod 2^32) that is subtracted once per word.
constexpr uint32_t kPack16Bias = (uint32_t)(0x4B400000ull * 0x55555555ull);   // sum over s<16 of kMagicBits << 2s
constexpr uint32_t kPack4Bias = (uint32_t)(0x4B400000ull * 0x01010101ull);    // sum over b<4 of kMagicBits << 8b

// TIERED: rows carry a tier and a source-row index (akvq_quantize_append_tiered); the plain instantiation is the
// two-bit path with identity row mapping and none of the per-row tier arithmetic.
// WINDOW: the last win_len appended rows also go to the recent-window rings.
// ROPE: K rows arrive without their rotary position embedding; it is applied here, in front of the rotation.
// (the tensor, 0 = K or 1 = V, is a template parameter of the body: the two differ in everything after the transform,
// and the kernel branches once, on blockIdx.z)
template <int G, bool TIERED, bool WINDOW, bool ROPE, int TENSOR>
__device__ __forceinline__ void quantize_append_body(const QuantArgs &a, int (*slot_of_lds)[kTokBlock],
                                                     uint32_t (*vtile_lds)[WINDOW ? 2048 : 4]) {
  // the wavefront index as a scalar: the block index, its first row and every base address derived from them then
  // live in scalar registers
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int blk_rel = blockIdx.x * 4 + wave;
  if (blk_rel >= a.n_blk) return;  // whole wavefront leaves; no block-wide barrier is used below
  const int blk = a.first_blk + blk_rel;
  const int bh = blockIdx.y;
  constexpr int tensor = TENSOR;
  const int r = lane >> 2, j = lane & 3;
  constexpr int NG = kD / G;

  const uint16_t *src = tensor == 0 ? a.k_new : a.v_new;
  const bool rotate = (tensor == 0 ? a.rotate_k : a.rotate_v) != 0;
  const float kappa = rotate ? inv_sqrt128() : 1.0f;
  const float lane_sign = rotate ? quad_sign(j) : 1.0f;  // this lane holds lane_sign * (transformed values)
  const float kappa_s = lane_sign * kappa;
  const int t0 = blk * kTokBlock;
  const int t_end = a.T_len + a.n_new;

  // ---- which tokens of this block are salient, and at which overlay slot (rank in the ascending list).
  // The list is ascending, so the block's entries are one contiguous run of at most 32.  Lane l samples entry
  // l*stride; the number of samples below the block start locates the run within one stride, and a second load of
  // 64 consecutive entries covers it.  Lists of up to 64 entries need the first load only.  Both loads are
  // independent of the row loads, which are issued in between so that all latencies overlap.
  int *slot_of = slot_of_lds[wave];
  const int32_t *sidx = a.sal_idx + (size_t)bh * a.S_cap;
  int cnt = a.sal_cnt[bh];
  cnt = min(max(cnt, 0), a.S_cap);
  const int stride = (cnt + 63) >> 6;
  int e1 = 0x7FFFFFFF;
  if (lane * stride < cnt) e1 = sidx[lane * stride];

  bool valid[2];
  int tier[2] = {AKVQ_TIER_2BIT, AKVQ_TIER_2BIT};
  u32x4 raw[2][4];
  u32x4 rope_c[ROPE ? 2 : 1][2], rope_s[ROPE ? 2 : 1][2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int t = t0 + 16 * h + r;
    valid[h] = (t >= a.T_len) && (t < t_end);
    // rows outside the appended range read a clamped (valid) address; nothing derived from them is stored
    const int rel = min(max(t - a.T_len, 0), a.n_new - 1);
    int src_row = rel;
    if constexpr (TIERED) {
      const size_t at = (size_t)(bh / a.Hkv) * a.n_new + rel;
      src_row = min(max(a.row_src[at], 0), a.n_src - 1);
      if (valid[h]) tier[h] = a.row_tier[at];
    }
    const uint16_t *row = src + ((size_t)bh * a.n_src + src_row) * kD;
#pragma unroll
    for (int m = 0; m < 4; ++m) raw[h][m] = *reinterpret_cast<const u32x4 *>(row + 32 * m + 8 * j);
    if constexpr (ROPE) {
      if (tensor == 0) {
        const size_t at = (size_t)(bh / a.Hkv) * a.rope_stride + (size_t)src_row * 64 + 8 * j;
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
          rope_c[h][mm] = *reinterpret_cast<const u32x4 *>(a.rope_cos + at + 32 * mm);
          rope_s[h][mm] = *reinterpret_cast<const u32x4 *>(a.rope_sin + at + 32 * mm);
        }
      }
    }
  }
  if constexpr (TIERED) {
    // fine-half mask of this block (one word per batch element): lane L < 32 looks at row t0 + L
    if (tensor == 0 && bh % a.Hkv == 0) {
      const int t = t0 + (lane & 31);
      const bool in_range = lane < kTokBlock && t >= a.T_len && t < t_end;
      const bool fine = in_range && a.row_tier[(size_t)(bh / a.Hkv) * a.n_new + (t - a.T_len)] == AKVQ_TIER_4BIT_FINE;
      const uint32_t written = (uint32_t)__ballot(in_range), bits = (uint32_t)__ballot(fine);
      if (lane == 0) {
        uint32_t *w = a.fine_mask + (size_t)(bh / a.Hkv) * (a.T_cap / kTokBlock) + blk;
        *w = (written == 0xFFFFFFFFu) ? bits : ((*w & ~written) | bits);
      }
    }
  }

  // A block that is only partly new (a decode step appends one row) keeps the other tokens' bits of its V words: the
  // words this lane will rewrite are requested now, with the rows, instead of after the arithmetic.
  const size_t blk_word = ((size_t)bh * (a.T_cap / kTokBlock) + blk) * kBlockWords;
  const bool partial_blk = t0 < a.T_len || t0 + kTokBlock > t_end;  // uniform over the wavefront
  u32x2 v_old[2] = {{0u, 0u}, {0u, 0u}};
  if (tensor == 1 && partial_blk) {
    const int ii = r & 3, q = r >> 2;
#pragma unroll
    for (int c = 0; c < 2; ++c)
      v_old[c] = *reinterpret_cast<const u32x2 *>(a.v_codes + blk_word + (size_t)(16 * q + 8 * (j & 1) + 2 * ii + c) * 4 +
                                                  2 * (j >> 1));
  }

  if (lane < kTokBlock) slot_of[lane] = -1;
  wave_lds_sync();
  if (stride <= 1) {
    if (e1 >= t0 && e1 < t0 + kTokBlock) slot_of[e1 - t0] = lane;
  } else if (stride <= 32) {
    const int below = __popcll(__ballot(e1 < t0));  // samples before the block: the run starts after the last of them
    const int idx = max(below - 1, 0) * stride + lane;
    const int e2 = idx < cnt ? sidx[idx] : 0x7FFFFFFF;
    if (e2 >= t0 && e2 < t0 + kTokBlock) slot_of[e2 - t0] = idx;
  } else {
    for (int base = 0; base < cnt; base += 64) {
      const int e = base + lane < cnt ? sidx[base + lane] : 0x7FFFFFFF;
      if (e >= t0 && e < t0 + kTokBlock) slot_of[e - t0] = base + lane;
    }
  }
  wave_lds_sync();

  // recent window: is this whole block new and inside the window?  (uniform over the wavefront)
  bool win_block = false;
  if constexpr (WINDOW) win_block = t0 >= a.T_len && t0 + kTokBlock <= t_end && t0 >= t_end - a.win_len;
  uint32_t kw[2][2];         // K words of token half h: [h][group-of-64 word]
  uint32_t vcode[2][8];      // V: [mpair][i]: raw patterns of (X, Y) x (half 0, half 1) in the four byte lanes
  uint32_t vmask_part = 0;
  uint32_t meta_out[2][NG];
  int slots[2];

#pragma unroll
  for (int h = 0; h < 2; ++h) {
    slots[h] = slot_of[16 * h + r];
    if (TIERED && tier[h] != AKVQ_TIER_2BIT) slots[h] = -1;  // only plain rows can be salient
    float u[4][8];  // lane_sign times the (rotated) row
    if constexpr (ROPE) {
      if (tensor == 0) rope_row_quad(raw[h], rope_c[h], rope_s[h]);
    }
    if (rotate) {
      wht128_quad(raw[h], u, j);
    } else {
#pragma unroll
      for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          u[m][2 * w] = half_bits_to_float(raw[h][m][w] & 0xFFFFu);
          u[m][2 * w + 1] = half_bits_to_float(raw[h][m][w] >> 16);
        }
    }

    // ---- bfloat16 copies: the overlay slot of a salient row (Section III-C.1: salient tokens keep 16-bit
    // precision) and the ring slot of a row inside the recent window (the last win_len appended rows) ----
    auto store_bf16_row = [&](uint16_t *k_rows, uint16_t *v_plane, int slot, bool token) {
      const float scale = kappa_s;
      if (tensor == 0) {
        uint16_t *dst = k_rows + (size_t)slot * kD;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          u32x4 o;
#pragma unroll
          for (int w = 0; w < 4; ++w)
            o[w] = token ? pack_bf16x2(scaled_row_value(u[m][2 * w], scale), scaled_row_value(u[m][2 * w + 1], scale)) : 0u;
          *reinterpret_cast<u32x4 *>(dst + 32 * m + 8 * j) = o;
        }
      } else {
        const int sb = slot >> 5, sh = (slot & 31) >> 4, sr = slot & 15, sq = sr >> 2, sii = sr & 3;
#pragma unroll
        for (int m = 0; m < 4; ++m)
#pragma unroll
          for (int i = 0; i < 8; ++i) {
            const int e = 32 * m + 8 * j + i, nb = e >> 4, n = e & 15;
            v_plane[(size_t)sb * 4096 + nb * 512 + (16 * sq + n) * 8 + 2 * sii + sh] =
                token ? (uint16_t)pack_bf16x2(scaled_row_value(u[m][i], scale), 0.0f) : (uint16_t)0;
          }
      }
    };
    if (valid[h] && slots[h] >= 0 && !a.skip_overlay)  // (long salient lists are stored by overlay_rows_kernel instead)
      store_bf16_row(a.k_sal + (size_t)bh * a.S_cap * kD, a.v_sal + (size_t)bh * a.S_cap * kD, slots[h], true);
    if constexpr (WINDOW) {
      const int t = t0 + 16 * h + r;
      // fine halves and padding rows carry no token: their ring slots are zeroed
      const bool token = !TIERED || (tier[h] != AKVQ_TIER_4BIT_FINE && tier[h] != AKVQ_TIER_PAD);
      if (win_block && tensor == 1) {
        // The whole block fills one 32-slot tile of the V ring (the prefill case).  In a tile the values of rows r and
        // r+16 of one channel are neighbours; this lane owns both rows and writes its 16-bit values into the wavefront's
        // tile in LDS, half 0 and then half 1, and the finished tile goes out as eight fully coalesced 1 KB stores.
        // (Scattered partial-line stores, as in the row-at-a-time path, are several times slower and would dominate the
        // tail of a prefill launch.)
        uint16_t *tile16 = reinterpret_cast<uint16_t *>(vtile_lds[wave]);
        const int sq = r >> 2, sii = r & 3;
#pragma unroll
        for (int m = 0; m < 4; ++m)
#pragma unroll
          for (int w = 0; w < 4; ++w) {
            const uint32_t pk = token ? pack_bf16x2(scaled_row_value(u[m][2 * w], kappa_s), scaled_row_value(u[m][2 * w + 1], kappa_s)) : 0u;
#pragma unroll
            for (int c = 0; c < 2; ++c) {
              const int e = 32 * m + 8 * j + 2 * w + c, nb = e >> 4, n = e & 15;
              tile16[nb * 512 + (16 * sq + n) * 8 + 2 * sii + h] = (uint16_t)(c == 0 ? pk : pk >> 16);
            }
          }
        if (h == 1) {
          // the tile goes to the ring (slot = row mod W, a multiple of 32 here)
          uint32_t *ring_out = reinterpret_cast<uint32_t *>(
              a.v_win + (size_t)bh * a.win_len * kD + (size_t)((t0 % max(a.win_len, 1)) >> 5) * 4096);
          wave_lds_sync();
#pragma unroll
          for (int x = 0; x < 8; ++x)
            *reinterpret_cast<u32x4 *>(ring_out + 256 * x + 4 * lane) =
                *reinterpret_cast<const u32x4 *>(vtile_lds[wave] + 256 * x + 4 * lane);
          wave_lds_sync();
        }
      }
      if (!(win_block && tensor == 1) && valid[h] && t >= t_end - a.win_len) {
        store_bf16_row(a.k_win + (size_t)bh * a.win_len * kD, a.v_win + (size_t)bh * a.win_len * kD,
                       t % max(a.win_len, 1), token);
      }
    }

    // ---- group extrema (quad reduction), scale, zero-point ----
    GroupQ gq[NG];
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      constexpr int MPG = 4 / NG;  // m-slices per group
      float mn = u[g * MPG][0], mx = u[g * MPG][0];
#pragma unroll
      for (int m = g * MPG; m < (g + 1) * MPG; ++m)
#pragma unroll
        for (int i = 0; i < 8; i += 2) minmax3(mn, mx, u[m][i], u[m][i + 1]);
      if (lane_sign < 0.0f) {  // extrema of the true values
        const float t = mn;
        mn = -mx;
        mx = -t;
      }
      quad_minmax(mn, mx);
      if constexpr (!TIERED) {
        gq[g] = group_params(mn, mx, kappa, a.clip, tier_two_bit());
        meta_out[h][g] = gq[g].meta | (slots[h] >= 0 ? 0x8000u : 0u);
      } else {
        const bool four = tier[h] == AKVQ_TIER_4BIT_COARSE || tier[h] == AKVQ_TIER_4BIT_FINE;
        const TierQ t2 = tier_two_bit(), t4 = tier_four_bit();
        const TierQ tq = {four ? t4.inv_levels : t2.inv_levels, four ? t4.s16_max : t2.s16_max};
        gq[g] = group_params(mn, mx, kappa, four ? a.clip4 : a.clip, tq);
        uint32_t mw = gq[g].meta | (slots[h] >= 0 ? 0x8000u : 0u);
        if (tier[h] == AKVQ_TIER_4BIT_COARSE)  // scale 4*s (exact in binary16), zero floor(z4 / 4)
          mw = float_to_half_bits_rne(4.0f * half_bits_to_float(gq[g].s16)) | ((uint32_t)((gq[g].z >> 2) & 0xFFFF) << 16);
        else if (tier[h] == AKVQ_TIER_4BIT_FINE)  // scale s, zero z4 mod 4
          mw = gq[g].s16 | ((uint32_t)(gq[g].z & 3) << 16);
        else if (tier[h] == AKVQ_TIER_PAD)  // ignored by decode: salient bit with scale bits 0, a marker no real row has
          mw = 0x8000u;
        meta_out[h][g] = mw;
      }
      gq[g].rcpu *= lane_sign;  // codes are taken from the signed values this lane holds
    }
    // per-row constants of the code extraction (tiered rows only)
    float code_top = kMagic + 3.0f;
    uint32_t code_shift = 0u, code_keep = 2u;  // field offset and width in bits
    if constexpr (TIERED) {
      if (tier[h] == AKVQ_TIER_4BIT_COARSE || tier[h] == AKVQ_TIER_4BIT_FINE) code_top = kMagic + 15.0f;
      if (tier[h] == AKVQ_TIER_4BIT_COARSE) code_shift = 2u;
      if (tier[h] == AKVQ_TIER_PAD) code_keep = 0u;
    }
    constexpr uint32_t kBias16 = TIERED ? 0u : kPack16Bias;
    auto row_code = [&](float x, const GroupQ &q) {
      if constexpr (TIERED) return code_bits_tiered(x, q, code_top, code_shift, code_keep);
      else return code_bits(x, q);
    };

    // ---- codes ----
    if (tensor == 0) {
      // K word (m/2): slot 8*(m%2)+i at bits 2*slot; built from the top slot down by shift-adds
#pragma unroll
      for (int wq = 0; wq < 2; ++wq) {
        uint32_t word = 0;
#pragma unroll
        for (int slot = 15; slot >= 0; --slot) {
          const int m = 2 * wq + (slot >> 3), i = slot & 7;
          word = (word << 2) + row_code(u[m][i], gq[m / (4 / NG)]);
          asm("" : "+v"(word));  // keep the chain one shift-add per code (re-association costs more instructions)
        }
        kw[h][wq] = word - kBias16;
      }
    } else {
      // V: byte lanes of a partial word: token half h, X (m even) / Y (m odd); biases removed after both halves
#pragma unroll
      for (int mp = 0; mp < 2; ++mp)
#pragma unroll
        for (int i = 0; i < 8; ++i) {
          const uint32_t bx = row_code(u[2 * mp][i], gq[(2 * mp) / (4 / NG)]);
          const uint32_t by = row_code(u[2 * mp + 1][i], gq[(2 * mp + 1) / (4 / NG)]);
          const uint32_t part = (by << 8) + bx;
          if (h == 0) vcode[mp][i] = part; else vcode[mp][i] = (part << 16) + vcode[mp][i];
        }
      if (valid[h]) vmask_part |= 0x0303u << (16 * h);
    }
  }

  // ---- meta ----
  if (j == 0) {
    uint32_t *meta = tensor == 0 ? a.k_meta : a.v_meta;
#pragma unroll
    for (int h = 0; h < 2; ++h)
      if (valid[h]) {
        uint32_t *dst = meta + ((size_t)bh * a.T_cap + t0 + 16 * h + r) * NG;
#pragma unroll
        for (int g = 0; g < NG; ++g) dst[g] = meta_out[h][g];
      }
  }

  if (tensor == 0) {
    // chunk 16*j + r: words {2h, 2h+1} belong to token half h
    uint32_t *chunk = a.k_codes + blk_word + (size_t)(16 * j + r) * 4;
    if (valid[0] && valid[1]) {
      u32x4 o = {kw[0][0], kw[0][1], kw[1][0], kw[1][1]};
      *reinterpret_cast<u32x4 *>(chunk) = o;
    } else if (valid[0]) {
      u32x2 o = {kw[0][0], kw[0][1]};
      *reinterpret_cast<u32x2 *>(chunk) = o;
    } else if (valid[1]) {
      u32x2 o = {kw[1][0], kw[1][1]};
      *reinterpret_cast<u32x2 *>(chunk + 2) = o;
    }
  } else {
    // shift the byte lanes to this token's pair position (ii = r%4), then OR over the four rows that share a chunk
    const int ii = r & 3, q = r >> 2;
    uint32_t mask = vmask_part << (2 * ii);
    mask |= dpp_move_u<kRowRor4>(mask);
    mask |= dpp_move_u<kRowRor8>(mask);
    if (mask != 0u) {  // uniform over the four rows of a chunk; in practice over the wavefront
      // all cross-lane work first, outside any divergent control flow: complete words of the lane's eight chunks
      uint32_t w[2][8];
#pragma unroll
      for (int i = 0; i < 8; ++i)
#pragma unroll
        for (int mp = 0; mp < 2; ++mp) {
          uint32_t x = (vcode[mp][i] - (TIERED ? 0u : kPack4Bias)) << (2 * ii);
          x |= dpp_move_u<kRowRor4>(x);
          x |= dpp_move_u<kRowRor8>(x);
          w[mp][i] = x;
        }
      // each of the four rows stores two of the eight chunks: i = 2*ii and 2*ii + 1
      uint32_t sel[2][2];
#pragma unroll
      for (int c = 0; c < 2; ++c)
#pragma unroll
        for (int mp = 0; mp < 2; ++mp) {
          uint32_t x = w[mp][c];
          x = ii == 1 ? w[mp][2 + c] : x;
          x = ii == 2 ? w[mp][4 + c] : x;
          x = ii == 3 ? w[mp][6 + c] : x;
          sel[c][mp] = x;
        }
#pragma unroll
      for (int c = 0; c < 2; ++c) {
        uint32_t *dst = a.v_codes + blk_word + (size_t)(16 * q + 8 * (j & 1) + 2 * ii + c) * 4 + 2 * (j >> 1);
        uint32_t w0 = sel[c][0], w1 = sel[c][1];
        if (mask != 0xFFFFFFFFu) {  // block only partly new: keep the other tokens' bits (read at the top)
          w0 = (v_old[c][0] & ~mask) | (w0 & mask);
          w1 = (v_old[c][1] & ~mask) | (w1 & mask);
        }
        u32x2 o = {w0, w1};
        *reinterpret_cast<u32x2 *>(dst) = o;
      }
    }
  }
}

template <int G, bool TIERED, bool WINDOW, bool ROPE>
__global__ __launch_bounds__(256) void quantize_append_kernel(QuantArgs a) {
  __shared__ int slot_of_lds[4][kTokBlock];
  __shared__ __attribute__((aligned(16))) uint32_t vtile_lds[WINDOW ? 4 : 1][WINDOW ? 2048 : 4];  // one V tile (32 slots x 128 channels, bf16) per wavefront
  if (blockIdx.z == 0) quantize_append_body<G, TIERED, WINDOW, ROPE, 0>(a, slot_of_lds, vtile_lds);
  else quantize_append_body<G, TIERED, WINDOW, ROPE, 1>(a, slot_of_lds, vtile_lds);
}

// ------------------------------------------------------------------------------------------------
// The 16-bit overlay rows of a long salient list (text-salient layers, Section III-B.1 / III-C.1), as a pass of their
// own behind the block kernel: one wavefront per 32-slot tile of the overlay and tensor.  It gathers the tile's rows
// through the salient list, transforms them exactly as the block kernel does (same butterflies, same roundings) and
// stores K rows whole and the V tile through LDS as eight coalesced 1 KB pieces, instead of one 2-byte store per value
// from whichever block a row happens to sit in.  Slots of the tile that are not being written (rows of earlier
// appends, unused slots) keep their contents: unless every slot is new the tile is read into LDS first.
// ------------------------------------------------------------------------------------------------
template <bool ROPE>
__global__ __launch_bounds__(256) void overlay_rows_kernel(QuantArgs a) {
  __shared__ __attribute__((aligned(16))) uint32_t vtile_lds[4][2048];
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int lane = threadIdx.x & 63;
  const int bh = blockIdx.y, tensor = blockIdx.z;
  const int s0 = (blockIdx.x * 4 + wave) * kTokBlock;
  const int cnt = min(max(a.sal_cnt[bh], 0), a.S_cap);
  if (s0 >= cnt) return;  // whole wavefront leaves; no block-wide barrier is used below
  const int r = lane >> 2, j = lane & 3;
  const int t_end = a.T_len + a.n_new;
  const uint16_t *src = tensor == 0 ? a.k_new : a.v_new;
  const bool rotate = (tensor == 0 ? a.rotate_k : a.rotate_v) != 0;
  const float kappa_s = rotate ? quad_sign(j) * inv_sqrt128() : 1.0f;
  const int32_t *sidx = a.sal_idx + (size_t)bh * a.S_cap;

  bool fresh[2];  // this lane's slot of half h holds a row of this append
  u32x4 raw[2][4];
  u32x4 rope_c[ROPE ? 2 : 1][2], rope_s[ROPE ? 2 : 1][2];
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int slot = s0 + 16 * h + r;
    const int t = slot < cnt ? sidx[slot] : -1;
    fresh[h] = t >= a.T_len && t < t_end;
    const int rel = min(max(t - a.T_len, 0), a.n_new - 1);  // other rows read a clamped (valid) address; nothing of them is stored
    const uint16_t *row = src + ((size_t)bh * a.n_src + rel) * kD;
#pragma unroll
    for (int m = 0; m < 4; ++m) raw[h][m] = *reinterpret_cast<const u32x4 *>(row + 32 * m + 8 * j);
    if constexpr (ROPE) {
      if (tensor == 0) {
        const size_t at = (size_t)(bh / a.Hkv) * a.rope_stride + (size_t)rel * 64 + 8 * j;
#pragma unroll
        for (int mm = 0; mm < 2; ++mm) {
          rope_c[h][mm] = *reinterpret_cast<const u32x4 *>(a.rope_cos + at + 32 * mm);
          rope_s[h][mm] = *reinterpret_cast<const u32x4 *>(a.rope_sin + at + 32 * mm);
        }
      }
    }
  }
  const unsigned long long n_fresh = __ballot(fresh[0]) | __ballot(fresh[1]);
  if (n_fresh == 0ull) return;  // a tile of earlier rows
  const bool all_fresh = __ballot(!fresh[0]) == 0ull && __ballot(!fresh[1]) == 0ull;
  uint32_t *tile_out = reinterpret_cast<uint32_t *>(a.v_sal + (size_t)bh * a.S_cap * kD + (size_t)(s0 >> 5) * 4096);
  if (tensor == 1 && !all_fresh) {
#pragma unroll
    for (int x = 0; x < 8; ++x)
      *reinterpret_cast<u32x4 *>(vtile_lds[wave] + 256 * x + 4 * lane) =
          *reinterpret_cast<const u32x4 *>(tile_out + 256 * x + 4 * lane);
    wave_lds_sync();
  }
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    float u[4][8];  // quad_sign(j) times the (rotated) row
    if constexpr (ROPE) {
      if (tensor == 0) rope_row_quad(raw[h], rope_c[h], rope_s[h]);
    }
    if (rotate) {
      wht128_quad(raw[h], u, j);
    } else {
#pragma unroll
      for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          u[m][2 * w] = half_bits_to_float(raw[h][m][w] & 0xFFFFu);
          u[m][2 * w + 1] = half_bits_to_float(raw[h][m][w] >> 16);
        }
    }
    if (tensor == 0) {
      if (fresh[h]) {
        uint16_t *dst = a.k_sal + ((size_t)bh * a.S_cap + s0 + 16 * h + r) * kD;
#pragma unroll
        for (int m = 0; m < 4; ++m) {
          u32x4 o;
#pragma unroll
          for (int w = 0; w < 4; ++w)
            o[w] = pack_bf16x2(scaled_row_value(u[m][2 * w], kappa_s), scaled_row_value(u[m][2 * w + 1], kappa_s));
          *reinterpret_cast<u32x4 *>(dst + 32 * m + 8 * j) = o;
        }
      }
    } else if (fresh[h]) {
      // in a tile the values of slots r and r + 16 of one channel are neighbours (see the recent-window tiles)
      uint16_t *tile16 = reinterpret_cast<uint16_t *>(vtile_lds[wave]);
      const int sq = r >> 2, sii = r & 3;
#pragma unroll
      for (int m = 0; m < 4; ++m)
#pragma unroll
        for (int w = 0; w < 4; ++w) {
          const uint32_t pk = pack_bf16x2(scaled_row_value(u[m][2 * w], kappa_s), scaled_row_value(u[m][2 * w + 1], kappa_s));
#pragma unroll
          for (int c = 0; c < 2; ++c) {
            const int e = 32 * m + 8 * j + 2 * w + c, nb = e >> 4, n = e & 15;
            tile16[nb * 512 + (16 * sq + n) * 8 + 2 * sii + h] = (uint16_t)(c == 0 ? pk : pk >> 16);
          }
        }
    }
  }
  if (tensor == 1) {
    wave_lds_sync();
#pragma unroll
    for (int x = 0; x < 8; ++x)
      *reinterpret_cast<u32x4 *>(tile_out + 256 * x + 4 * lane) =
          *reinterpret_cast<const u32x4 *>(vtile_lds[wave] + 256 * x + 4 * lane);
  }
}

template <int G>
__global__ __launch_bounds__(64) void append_row_kernel(QuantArgs a) {
  __shared__ __attribute__((aligned(16))) uint8_t code_lds[kD];
  __shared__ __attribute__((aligned(16))) uint16_t row_lds[kD];
  append_row_wave<G>(a, blockIdx.x, blockIdx.y, threadIdx.x, code_lds, row_lds);
}

}  // namespace

static void launch_blocks(const QuantArgs &a, int B, int G, bool window, hipStream_t stream) {
  dim3 grid((a.n_blk + 3) / 4, B * a.Hkv, 2), block(256);
  const bool tiered = a.row_tier != nullptr;
  const bool rope = a.rope_cos != nullptr;
#define AKVQ_LAUNCH_Q(GG, TT, WW, RR) \
  hipLaunchKernelGGL((quantize_append_kernel<GG, TT, WW, RR>), grid, block, 0, stream, a)
#define AKVQ_LAUNCH_QR(GG, TT, WW) \
  do { if (rope) AKVQ_LAUNCH_Q(GG, TT, WW, true); else AKVQ_LAUNCH_Q(GG, TT, WW, false); } while (0)
  if (G == 128) {
    if (tiered) { if (window) AKVQ_LAUNCH_QR(128, true, true); else AKVQ_LAUNCH_QR(128, true, false); }
    else { if (window) AKVQ_LAUNCH_QR(128, false, true); else AKVQ_LAUNCH_QR(128, false, false); }
  } else {
    if (tiered) { if (window) AKVQ_LAUNCH_QR(64, true, true); else AKVQ_LAUNCH_QR(64, true, false); }
    else { if (window) AKVQ_LAUNCH_QR(64, false, true); else AKVQ_LAUNCH_QR(64, false, false); }
  }
#undef AKVQ_LAUNCH_QR
#undef AKVQ_LAUNCH_Q
}

static hipError_t launch_block_ranges(const QuantArgs &a, int B, int G, hipStream_t stream);

hipError_t launch_quantize_append(const QuantArgs &a, int B, int G, hipStream_t stream) {
  if (a.n_new == 1 && a.n_src == 1 && a.row_tier == nullptr) {  // the decode step: one plain row per (batch, kv-head)
    dim3 grid(B * a.Hkv, 2), block(64);
    if (G == 128) hipLaunchKernelGGL(append_row_kernel<128>, grid, block, 0, stream, a);
    else hipLaunchKernelGGL(append_row_kernel<64>, grid, block, 0, stream, a);
    return hipGetLastError();
  }
  // Long salient lists (text-salient layers) get their overlay rows from a pass of their own behind the block kernel;
  // a handful of pivots (and the rows of a tiered append, whose tiers the block kernel knows) are stored by the block
  // kernel itself.
  if (a.S_cap > 64 && a.row_tier == nullptr) {
    QuantArgs blocks = a;
    blocks.skip_overlay = 1;
    hipError_t e = launch_block_ranges(blocks, B, G, stream);
    if (e != hipSuccess) return e;
    dim3 grid((a.S_cap / kTokBlock + 3) / 4, B * a.Hkv, 2), block(256);
    if (a.rope_cos != nullptr) hipLaunchKernelGGL(overlay_rows_kernel<true>, grid, block, 0, stream, a);
    else hipLaunchKernelGGL(overlay_rows_kernel<false>, grid, block, 0, stream, a);
    return hipGetLastError();
  }
  return launch_block_ranges(a, B, G, stream);
}

hipError_t launch_block_ranges(const QuantArgs &a, int B, int G, hipStream_t stream) {
  if (a.win_len <= 0) {
    launch_blocks(a, B, G, false, stream);
    return hipGetLastError();
  }
  // Recent window: only the blocks that hold the last win_len new rows write ring slots.  A long append (prefill)
  // runs the plain instantiation over the blocks before them, so that the ring stores (and the registers and LDS
  // they need) stay out of the bulk of the work, then the windowed instantiation over the few window blocks.
  const int t_end = a.T_len + a.n_new;
  const int t_w0 = t_end - a.win_len > a.T_len ? t_end - a.win_len : a.T_len;
  const int win_first_blk = t_w0 / kTokBlock;
  if (win_first_blk > a.first_blk) {
    QuantArgs head = a;
    head.n_blk = win_first_blk - a.first_blk;
    head.win_len = 0;
    launch_blocks(head, B, G, false, stream);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
  }
  QuantArgs tail = a;
  tail.first_blk = win_first_blk;
  tail.n_blk = a.first_blk + a.n_blk - win_first_blk;
  launch_blocks(tail, B, G, true, stream);
  return hipGetLastError();
}

}  // namespace akvq

// Device-side helpers shared by the gfx950 kernels of libakvq (number formats, wave-level primitives,
// matrix-core operand types, the 2-bit -> bfloat16 operand expansion).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

namespace akvq {

constexpr int kD = 128;          // head_dim
constexpr int kWave = 64;        // wavefront width on CDNA4
constexpr int kTokBlock = 32;    // tokens per cache block (1024 bytes of codes)
constexpr int kBlockWords = 256; // uint32 words per block

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

// 2^-3.5: the normalisation of the 128-point Walsh-Hadamard matrix (seven levels of 1/sqrt(2), Eq. 7).
__device__ __forceinline__ float inv_sqrt128() { return __uint_as_float(0x3DB504F3u); }

__device__ __forceinline__ float half_bits_to_float(uint32_t h16) {
  return (float)__builtin_bit_cast(_Float16, (unsigned short)h16);
}
// float -> binary16 bits, round to nearest even (the conversion instruction's default mode)
__device__ __forceinline__ uint32_t float_to_half_bits_rne(float f) {
  return (uint32_t)__builtin_bit_cast(unsigned short, (_Float16)f);
}

// float -> bfloat16 bits, round to nearest even (finite inputs).
__device__ __forceinline__ uint32_t f32_to_bf16_rne(float f) {
  uint32_t u = __float_as_uint(f);
  u += 0x7FFFu + ((u >> 16) & 1u);
  return u >> 16;
}
__device__ __forceinline__ float bf16_bits_to_f32(uint32_t b) { return __uint_as_float(b << 16); }
// two floats -> packed bfloat16 pair (lo = a, hi = b), round to nearest even, one conversion instruction
__device__ __forceinline__ uint32_t pack_bf16x2(float a, float b) {
  typedef __attribute__((ext_vector_type(2))) float f32x2_t;
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2_t;
  f32x2_t v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Split a float into up to three bfloat16 terms whose sum reproduces it to ~24 bits.
__device__ __forceinline__ void split3_bf16(float v, uint32_t &hi, uint32_t &mid, uint32_t &lo) {
  hi = f32_to_bf16_rne(v);
  float r1 = v - bf16_bits_to_f32(hi);
  mid = f32_to_bf16_rne(r1);
  float r2 = r1 - bf16_bits_to_f32(mid);
  lo = f32_to_bf16_rne(r2);
}

// Load of data that is read once per launch (the cache stream of decode, the hidden states of the massive-activation
// score): the non-temporal hint keeps such lines from being retained in the cache hierarchy.  Measured on a plain
// 2 GiB streaming read of 128-bit loads: 7.1 TB/s with the hint against 6.3 TB/s without; decode at B=64, T=8192 went
// from 71 % to 78 % of the HBM peak.  The write path and the pivot score (bound by instruction issue, not by memory)
// measured no gain and keep plain loads.
template <typename T>
__device__ __forceinline__ T stream_load(const T *p) { return __builtin_nontemporal_load(p); }

// Pointers into the cache stream are kept as explicit global-memory pointers.  keep_scalar pins a wavefront-uniform
// one in scalar registers, so that "pointer + per-lane offset" is issued as a load with a scalar base and a 32-bit lane
// offset instead of being re-associated into per-lane 64-bit arithmetic (the address space has to be explicit because
// the compiler cannot see through the pin).
#define AKVQ_GLOBAL __attribute__((address_space(1)))
typedef const AKVQ_GLOBAL uint32_t *gptr_u32;
__device__ __forceinline__ gptr_u32 as_global(const uint32_t *p) { return (gptr_u32)p; }
__device__ __forceinline__ void keep_scalar(gptr_u32 &p) { asm volatile("" : "+s"(p)); }
__device__ __forceinline__ u32x4 stream_load_x4(gptr_u32 p) { return __builtin_nontemporal_load((const AKVQ_GLOBAL u32x4 *)p); }
__device__ __forceinline__ u32x2 stream_load_x2(gptr_u32 p) { return __builtin_nontemporal_load((const AKVQ_GLOBAL u32x2 *)p); }
__device__ __forceinline__ uint32_t stream_load_x1(gptr_u32 p) { return __builtin_nontemporal_load(p); }

// Make the compiler treat these registers as consumed here, so that any load filling them is waited for at this
// point.  Used once before a software-pipelined loop: the loop header then starts with no load outstanding, and the
// waits inside the loop count only the loads of the tile being prefetched (otherwise the first-iteration state makes
// every iteration wait for its own prefetch right after issuing it).
__device__ __forceinline__ void settle(u32x4 &v) { asm volatile("" : "+v"(v)); }
__device__ __forceinline__ void settle(uint32_t &v) { asm volatile("" : "+v"(v)); }

// ---- wave-level reductions (64 lanes) ----
__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v = fmaxf(v, __shfl_xor(v, off, kWave));
  return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) v += __shfl_xor(v, off, kWave);
  return v;
}

// LDS traffic between lanes of one wavefront needs no hardware wait: a wavefront's LDS instructions execute in
// issue order, so a read issued after a write sees it.  What is needed is that the compiler keeps that order (the
// memory clobber) and does not move code across (the wave barrier).  A release/acquire fence is deliberately NOT
// used here: it would also drain every outstanding global load, i.e. the prefetch of the next tiles.
__device__ __forceinline__ void wave_lds_sync() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_wave_barrier();
  asm volatile("" ::: "memory");
}

// ---- 2-bit codes -> bfloat16 matrix-core operands --------------------------------------------------
// A 32-bit code word holds 8 code pairs: pair p = (bits [2p,2p+2), bits [16+2p,16+2p+2)).
// OR-ing a masked pair into 0x4300'4300 yields two bfloat16 numbers 128 + 4^k * code (k = the field's
// position inside the 7-bit mantissa: 0, 1 or 2).  The constant 128 and the factor 4^k are undone on the
// other operand of the contraction, so expansion costs one and-or per two codes (plus two shifts per word).
// Pairs 0..3 form the "X" operand, pairs 4..7 the "Y" operand; both carry the factors 4^{0,1,2,0}.
// The masks and the constant are kept as opaque register values (not literals) so that the compiler selects the
// three-operand and-or instruction, whose encoding takes no literal operands: D = (w & mask) | magic in one op.
struct ExpandK {
  uint32_t magic;    // 0x4300'4300, vector register
  uint32_t mask[3];  // 0x0003'0003 << {0,2,4}, scalar registers
  __device__ __forceinline__ ExpandK() {
    uint32_t m = 0x43004300u, m0 = 0x00030003u, m1 = 0x000C000Cu, m2 = 0x00300030u;
    asm volatile("" : "+v"(m), "+s"(m0), "+s"(m1), "+s"(m2));
    magic = m; mask[0] = m0; mask[1] = m1; mask[2] = m2;
  }
  __device__ __forceinline__ uint32_t pair(uint32_t w, int k) const { return (w & mask[k]) | magic; }
  __device__ __forceinline__ bf16x8 x(uint32_t w) const {
    const uint32_t w6 = w >> 6;
    u32x4 r = {pair(w, 0), pair(w, 1), pair(w, 2), pair(w6, 0)};
    return __builtin_bit_cast(bf16x8, r);
  }
  __device__ __forceinline__ bf16x8 y(uint32_t w) const {
    const uint32_t w8 = w >> 8, w14 = w >> 14;
    u32x4 r = {pair(w8, 0), pair(w8, 1), pair(w8, 2), pair(w14, 0)};
    return __builtin_bit_cast(bf16x8, r);
  }
};
// exponent k (factor 4^k) carried by pair i of either operand: {0,1,2,0} (the Y operand shifts by 8 and 14 so that
// it repeats the X pattern; one set of pre-divided weights then serves both)
__device__ __forceinline__ int pair_exp(int i) { return i == 3 ? 0 : i; }
constexpr float kCodeBias = 128.0f; // the 2^7 every expanded code carries

typedef __attribute__((ext_vector_type(4))) int i32x4;
// 16x16x64 int8 product: per lane 16 K-slots (4 registers x 4 bytes); exact int32 accumulation
__device__ __forceinline__ i32x4 mfma_i8(i32x4 a, i32x4 b, i32x4 c) {
  return __builtin_amdgcn_mfma_i32_16x16x64_i8(a, b, c, 0, 0, 0);
}
// 16 two-bit codes of one word -> 16 int8 values (register j, byte b = code slot 4b + j): three shifts, four ands
struct ExpandI8 {
  uint32_t mask;  // 0x03030303 in a scalar register
  __device__ __forceinline__ ExpandI8() {
    uint32_t m = 0x03030303u;
    asm volatile("" : "+s"(m));
    mask = m;
  }
  __device__ __forceinline__ i32x4 operator()(uint32_t w) const {
    u32x4 r = {w & mask, (w >> 2) & mask, (w >> 4) & mask, (w >> 6) & mask};
    return __builtin_bit_cast(i32x4, r);
  }
};

__device__ __forceinline__ f32x4 mfma_bf16(bf16x8 a, bf16x8 b, f32x4 c) {
  return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
}

} // namespace akvq

// qkv_encode.h — device helpers shared by the kernels that write a card: the quantizer of one span of
// 32 values (group extrema, scale, reciprocal, codes) and the card stores.  Internal to the GPU library.
#pragma once

#include "qkv_common.h"
#include "qkv_decode.h"

namespace qkv {

// ---- small wrappers around instructions the compiler does not pick by itself ---------------

template <int CTRL>
__device__ inline uint32_t dpp(uint32_t v) {
  return (uint32_t)__builtin_amdgcn_update_dpp(0, (int)v, CTRL, 0xF, 0xF, false);
}
constexpr int kQuadXor1 = 0xB1;        // quad_perm:[1,0,3,2]
constexpr int kQuadXor2 = 0x4E;        // quad_perm:[2,3,0,1]

__device__ inline uint32_t pk_min3(uint32_t a, uint32_t b, uint32_t c) {
  uint32_t r;
  asm("v_pk_minimum3_f16 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
__device__ inline uint32_t pk_max3(uint32_t a, uint32_t b, uint32_t c) {
  uint32_t r;
  asm("v_pk_maximum3_f16 %0, %1, %2, %3" : "=v"(r) : "v"(a), "v"(b), "v"(c));
  return r;
}
__device__ inline uint32_t pk_min(uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_pk_min_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
__device__ inline uint32_t pk_max(uint32_t a, uint32_t b) {
  uint32_t r;
  asm("v_pk_max_f16 %0, %1, %2" : "=v"(r) : "v"(a), "v"(b));
  return r;
}
// both halves <- min / max of the two halves
__device__ inline uint32_t pk_min_halves(uint32_t a) {
  uint32_t r;
  asm("v_pk_min_f16 %0, %1, %1 op_sel:[0,1] op_sel_hi:[1,0]" : "=v"(r) : "v"(a));
  return r;
}
__device__ inline uint32_t pk_max_halves(uint32_t a) {
  uint32_t r;
  asm("v_pk_max_f16 %0, %1, %1 op_sel:[0,1] op_sel_hi:[1,0]" : "=v"(r) : "v"(a));
  return r;
}
// f32(low half of w) + c and f32(high half of w) + c: conversion and addition in one
// instruction, the sum rounded once to fp32
__device__ inline float lo_plus(uint32_t w, float c) {
  float r;
  asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(w), "v"(c));
  return r;
}
__device__ inline float hi_plus(uint32_t w, float c) {
  float r;
  asm("v_fma_mix_f32 %0, %1, 1.0, %2 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(r) : "v"(w), "v"(c));
  return r;
}

// (a << s) + b in one instruction
__device__ inline uint32_t shl_add(uint32_t a, uint32_t s, uint32_t b) {
  uint32_t r;
  asm("v_lshl_add_u32 %0, %1, %2, %3" : "=v"(r) : "v"(a), "n"(s), "v"(b));
  return r;
}

__device__ inline uint32_t float_to_half_bits(float f) {
  return (uint32_t)__builtin_bit_cast(uint16_t, (_Float16)f);   // round to nearest even
}

constexpr float kMagic = 12582912.0f;       // 2^23 + 2^22: adding it rounds to an integer, ties to even
constexpr uint32_t kMagicBits = 0x4B400000u;

// Sum of kMagicBits << (i*W) over the 32/W codes that share one 32-bit accumulator.
template <int W>
__host__ __device__ constexpr uint32_t magic_carry() {
  uint32_t s = 0;
  for (int i = 0; i < 32 / W; ++i) s += kMagicBits << (i * W);
  return s;
}

// Card stores.  KEEP: plain stores, the card stays in the memory-side cache for a receiver
// that unpacks it next; otherwise nontemporal, for cards far larger than that cache.
template <bool KEEP, typename V>
__device__ inline void card_store(V* p, V v) {
  if (KEEP) *p = v; else __builtin_nontemporal_store(v, p);
}

template <int W, bool CLAMP>
__device__ inline void encode_span(const uint32_t (&w)[16], float neg_mn, float inv, uint32_t (&out)[W]) {
  constexpr uint32_t QMAX = (1u << W) - 1u;
  constexpr int PER = 32 / W;               // codes per output dword
#pragma unroll
  for (int i = 0; i < 32; ++i) {
    const float d = (i & 1) ? hi_plus(w[i >> 1], neg_mn) : lo_plus(w[i >> 1], neg_mn);
    const float r = __builtin_fmaf(d, inv, kMagic);       // exact product, one rounding, ties to even
    uint32_t u = __float_as_uint(r);
    if (CLAMP) u = min(u, kMagicBits + QMAX);
    const int o = i / PER, s = (i % PER) * W;
    out[o] = (s == 0) ? u : shl_add(u, s, out[o]);
  }
#pragma unroll
  for (int o = 0; o < W; ++o) out[o] -= magic_carry<W>();
}

// One span of 32 values (16 packed pairs): the extrema of its group (reduced over the GS lanes that share
// it), scale and reciprocal as the quantizer defines them, and the span's codes.  Returns the pair as it
// is stored: fp16 scale, then fp16 zero.
template <int W, int GS>
__device__ inline uint32_t quantize_span(const uint32_t (&w)[16], uint32_t (&out)[W]) {
  constexpr float QMAXF = (float)((1 << W) - 1);
  constexpr float RCPQ = 1.0f / QMAXF;           // correctly rounded at compile time
  // extrema of the span, then of the group
  uint32_t m = pk_min(pk_min3(pk_min3(w[0], w[1], w[2]), pk_min3(w[3], w[4], w[5]), pk_min3(w[6], w[7], w[8])),
                      pk_min3(pk_min3(w[9], w[10], w[11]), pk_min3(w[12], w[13], w[14]), w[15]));
  uint32_t M = pk_max(pk_max3(pk_max3(w[0], w[1], w[2]), pk_max3(w[3], w[4], w[5]), pk_max3(w[6], w[7], w[8])),
                      pk_max3(pk_max3(w[9], w[10], w[11]), pk_max3(w[12], w[13], w[14]), w[15]));
  m = pk_min_halves(m);
  M = pk_max_halves(M);
  if (GS >= 2) { m = pk_min(m, dpp<kQuadXor1>(m)); M = pk_max(M, dpp<kQuadXor1>(M)); }
  if (GS >= 4) { m = pk_min(m, dpp<kQuadXor2>(m)); M = pk_max(M, dpp<kQuadXor2>(M)); }
  const uint32_t mn_h = m & 0xFFFFu;

  // scale = fp16(range / qmax), inv = 1 / scale: fp32, correctly rounded.
  // Quotient: q0 = range * (1/qmax) is within one ulp, its exact residual corrects it.
  const float fmn = half_bits_to_float(mn_h);
  const float fmx = half_bits_to_float(M & 0xFFFFu);
  const float range = fmx - fmn;
  const float q0 = range * RCPQ;
  float s32 = __builtin_fmaf(__builtin_fmaf(-q0, QMAXF, range), RCPQ, q0);
  // Keep the fp32 quotient and its conversion apart: fused into one fma-and-convert
  // instruction the value would be rounded once, straight to fp16, which differs from
  // rounding to fp32 first whenever the fp32 result lands on an fp16 midpoint.
  asm("" : "+v"(s32));
  const uint32_t s_h = float_to_half_bits(s32);
  const float s = half_bits_to_float(s_h);
  // Reciprocal: the hardware estimate is within one ulp; s has 11 significant bits, so 1/s
  // is never closer than 2^-12 ulp to a rounding boundary and one residual step lands on
  // the correctly rounded value.
  const float y0 = __builtin_amdgcn_rcpf(s);
  const float y1 = __builtin_fmaf(__builtin_fmaf(-s, y0, 1.0f), y0, y0);
  const float inv = (s > 0.0f) ? y1 : 0.0f;

  // The clamp to qmax can only act when the stored scale is an fp16 subnormal; otherwise
  // d * inv <= qmax * (1 + 2^-11 + ...) already rounds to at most qmax.
  const bool needs_clamp = (s_h - 1u) < 0x3FFu;
  if (__builtin_amdgcn_ballot_w64(needs_clamp) != 0) encode_span<W, true>(w, -fmn, inv, out);
  else encode_span<W, false>(w, -fmn, inv, out);
  return s_h | (mn_h << 16);
}

}  // namespace qkv

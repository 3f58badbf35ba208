// qkv_decode.h — device helpers shared by the kernels that read a card: header validation
// and the decoder of one span of 32 values.  Internal to the GPU library.
#pragma once

#include <cstddef>

#include "qkv_common.h"

namespace qkv {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef float f32x2 __attribute__((ext_vector_type(2)));

__device__ inline float half_bits_to_float(uint32_t h) {
  return (float)__builtin_bit_cast(_Float16, (uint16_t)h);
}

// Card loads.  KEEP: plain loads, which find a card that was packed a moment ago in the
// memory-side cache; otherwise nontemporal, for cards far larger than that cache.
template <bool KEEP, typename V>
__device__ inline V card_load(const V* p) {
  return KEEP ? *p : __builtin_nontemporal_load(p);
}

// True when the header describes a layout-v1 card of the expected shape and grouping (flags word) that
// fits in card_bytes; fills `g` from the header's class counts.  Uniform over the grid.
//
// Every wave of every kernel that reads a card starts here, so the latency of this function is
// on the critical path of the first waves: the header's first 192 bytes are fetched as one batch
// of loads from a uniform address (the field offsets are those of qkv_card_header_t), and the
// checks are plain and-ed comparisons with a single branch, instead of a chain of short-circuit
// tests that would each wait for its own load.
__device__ inline bool card_geometry_from_header(const uint8_t* card, uint64_t card_bytes, uint32_t layers,
                                                 uint32_t kv_heads, uint32_t head_dim, uint32_t group_size,
                                                 uint64_t tokens, CardGeom& g, uint32_t want_flags = 0u) {
  static_assert(offsetof(qkv_card_header_t, version) == 8 && offsetof(qkv_card_header_t, tokens) == 32 &&
                offsetof(qkv_card_header_t, count) == 40 && offsetof(qkv_card_header_t, total_bytes) == 72 &&
                offsetof(qkv_card_header_t, off_bits) == 80 && offsetof(qkv_card_header_t, off_codes) == 104 &&
                offsetof(qkv_card_header_t, off_meta) == 128 && offsetof(qkv_card_header_t, off_fp16) == 152 &&
                offsetof(qkv_card_header_t, flags) == 188, "word indices below follow the header's layout");
  const uint32_t* w = reinterpret_cast<const uint32_t*>(card);
  uint32_t hw[48];
#pragma unroll
  for (int i = 0; i < 48; ++i) hw[i] = w[i];
  const auto u64_at = [&hw](int word) { return (uint64_t)hw[word] | ((uint64_t)hw[word + 1] << 32); };
  uint32_t ok = (uint32_t)(hw[0] == 0x43564B51u) & (uint32_t)(hw[1] == 0x00445241u);          // "QKVC" "ARD\0"
  ok &= (uint32_t)(hw[2] == QKV_CARD_VERSION) & (uint32_t)(hw[3] == QKV_CARD_HEADER_BYTES) & (uint32_t)(hw[47] == want_flags);
  ok &= (uint32_t)(hw[4] == layers) & (uint32_t)(hw[5] == kv_heads) & (uint32_t)(hw[6] == head_dim) &
        (uint32_t)(hw[7] == group_size) & (uint32_t)(u64_at(8) == tokens);
  uint64_t counts[4];
  uint64_t sum = 0;
#pragma unroll
  for (int c = 0; c < 4; ++c) {
    counts[c] = u64_at(10 + 2 * c);
    ok &= (uint32_t)(counts[c] <= tokens);       // with every count bounded the sum cannot wrap
    sum += counts[c];
  }
  ok &= (uint32_t)(sum == tokens);
  if (!ok) return false;
  build_geom(g, layers, kv_heads, head_dim, group_size, tokens, counts);
  ok = (uint32_t)(g.total <= card_bytes) & (uint32_t)(u64_at(18) == g.total);
  ok &= (uint32_t)(u64_at(20) == g.off_bits) & (uint32_t)(u64_at(22) == g.off_slot) & (uint32_t)(u64_at(24) == g.off_order) &
        (uint32_t)(u64_at(38) == g.off_fp16);
#pragma unroll
  for (int c = 0; c < 3; ++c)
    ok &= (uint32_t)(u64_at(26 + 2 * c) == g.off_codes[c]) & (uint32_t)(u64_at(32 + 2 * c) == g.off_meta[c]);
  return ok != 0u;
}

// decode = fp16( fma(code, scale, zero) ): an fp32 fma rounded to fp32, then rounded to
// fp16, both to nearest even.  The two steps are kept apart on purpose: the fused
// fma-and-convert instruction rounds the exact sum once, straight to fp16, which gives a
// different value whenever the fp32 result lands on an fp16 midpoint.
__device__ inline uint32_t decode_pair(float q0, float q1, float s, float z) {
  float a = __builtin_fmaf(q0, s, z);
  float b = __builtin_fmaf(q1, s, z);
  asm("" : "+v"(a));
  asm("" : "+v"(b));
  const f32x2 v = {a, b};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2));
}

// float(byte j of w): one instruction
__device__ inline float byte_to_float(uint32_t w, int j) {
  float r;
  switch (j) {
    case 0: asm("v_cvt_f32_ubyte0 %0, %1" : "=v"(r) : "v"(w)); break;
    case 1: asm("v_cvt_f32_ubyte1 %0, %1" : "=v"(r) : "v"(w)); break;
    case 2: asm("v_cvt_f32_ubyte2 %0, %1" : "=v"(r) : "v"(w)); break;
    default: asm("v_cvt_f32_ubyte3 %0, %1" : "=v"(r) : "v"(w)); break;
  }
  return r;
}

// The 32 values of one span: W dwords of codes in, 16 dwords of packed fp16 out.
template <int W>
__device__ inline void decode_span(const uint32_t (&cw)[W], float s, float z, uint32_t (&out)[16]) {
  if (W == 8) {
#pragma unroll
    for (int d = 0; d < 8; ++d) {          // dword d: codes 4d .. 4d+3, one per byte
      out[2 * d] = decode_pair(byte_to_float(cw[d], 0), byte_to_float(cw[d], 1), s, z);
      out[2 * d + 1] = decode_pair(byte_to_float(cw[d], 2), byte_to_float(cw[d], 3), s, z);
    }
  } else if (W == 4) {
#pragma unroll
    for (int d = 0; d < 4; ++d) {          // dword d: codes 8d .. 8d+7; byte j holds codes 2j (low), 2j+1 (high)
      const uint32_t even = cw[d] & 0x0F0F0F0Fu, odd = (cw[d] >> 4) & 0x0F0F0F0Fu;
#pragma unroll
      for (int j = 0; j < 4; ++j) out[4 * d + j] = decode_pair(byte_to_float(even, j), byte_to_float(odd, j), s, z);
    }
  } else {
#pragma unroll
    for (int d = 0; d < 2; ++d) {          // dword d: codes 16d .. 16d+15; byte j holds codes 4j .. 4j+3
      const uint32_t c0 = cw[d] & 0x03030303u, c1 = (cw[d] >> 2) & 0x03030303u, c2 = (cw[d] >> 4) & 0x03030303u,
                     c3 = (cw[d] >> 6) & 0x03030303u;
#pragma unroll
      for (int j = 0; j < 4; ++j) {
        out[8 * d + 2 * j] = decode_pair(byte_to_float(c0, j), byte_to_float(c1, j), s, z);
        out[8 * d + 2 * j + 1] = decode_pair(byte_to_float(c2, j), byte_to_float(c3, j), s, z);
      }
    }
  }
}

// 2-bit spans decoded by selection instead of arithmetic: a group has only four decoded values
// x_k = fp16(fma(k, scale, zero)), computed once per span; a table in LDS, indexed by a byte of
// four codes, holds the two byte selectors that pick (x_c0, x_c1) and (x_c2, x_c3) out of the
// eight bytes {x_0 .. x_3}.  About one vector instruction per value instead of three.
__device__ inline void build_select_table(u32x2* table, uint32_t lane) {
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const uint32_t b = lane * 4u + i;
    const uint32_t c0 = b & 3u, c1 = (b >> 2) & 3u, c2 = (b >> 4) & 3u, c3 = b >> 6;
    table[b] = (u32x2){0x01000100u + 2u * (c0 * 0x0101u + c1 * 0x01010000u),
                       0x01000100u + 2u * (c2 * 0x0101u + c3 * 0x01010000u)};
  }
}

// 8 * (byte J of w), the offset of a byte's entry in the selector table: one instruction (a shift whose
// operand is picked out of the register by sub-dword addressing) instead of an extraction and a shift.
template <int J>
__device__ inline uint32_t byte_times8(uint32_t w) {
  uint32_t r;
  const uint32_t three = 3u;
  if (J == 0) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_0" : "=v"(r) : "v"(three), "v"(w));
  if (J == 1) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_1" : "=v"(r) : "v"(three), "v"(w));
  if (J == 2) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_2" : "=v"(r) : "v"(three), "v"(w));
  if (J == 3) asm("v_lshlrev_b32_sdwa %0, %1, %2 dst_sel:DWORD dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:BYTE_3" : "=v"(r) : "v"(three), "v"(w));
  return r;
}

// The 32 values of a 2-bit span through the selector table (given as its first byte): same values as decode_span<2>.
__device__ inline void decode_span2_select(const uint32_t (&cw)[2], float s, float z, const uint8_t* table,
                                           uint32_t (&out)[16]) {
  const uint32_t x01 = decode_pair(0.0f, 1.0f, s, z);
  const uint32_t x23 = decode_pair(2.0f, 3.0f, s, z);
#pragma unroll
  for (int w = 0; w < 2; ++w) {
    const u32x2 sel0 = *reinterpret_cast<const u32x2*>(table + byte_times8<0>(cw[w]));
    const u32x2 sel1 = *reinterpret_cast<const u32x2*>(table + byte_times8<1>(cw[w]));
    const u32x2 sel2 = *reinterpret_cast<const u32x2*>(table + byte_times8<2>(cw[w]));
    const u32x2 sel3 = *reinterpret_cast<const u32x2*>(table + byte_times8<3>(cw[w]));
    out[8 * w + 0] = __builtin_amdgcn_perm(x23, x01, sel0.x);
    out[8 * w + 1] = __builtin_amdgcn_perm(x23, x01, sel0.y);
    out[8 * w + 2] = __builtin_amdgcn_perm(x23, x01, sel1.x);
    out[8 * w + 3] = __builtin_amdgcn_perm(x23, x01, sel1.y);
    out[8 * w + 4] = __builtin_amdgcn_perm(x23, x01, sel2.x);
    out[8 * w + 5] = __builtin_amdgcn_perm(x23, x01, sel2.y);
    out[8 * w + 6] = __builtin_amdgcn_perm(x23, x01, sel3.x);
    out[8 * w + 7] = __builtin_amdgcn_perm(x23, x01, sel3.y);
  }
}

}  // namespace qkv

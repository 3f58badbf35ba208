// qkv_plan.h — device helpers shared by the kernels that write a card's front matter (header,
// bits / slot / order tables, section pads; paper Sec. 4.2.1: the metadata a card carries).
// Internal to the GPU library.
#pragma once

#include "qkv_common.h"

namespace qkv {

// Class of a width: 4 -> 1, 8 -> 2, 16 -> 3, everything else 0 (2, and also invalid widths, which
// are flagged in the header: order[] stays a permutation and every index stays in range).
__device__ inline uint32_t class_of(uint32_t b) { return (b == 4) ? 1u : (b == 8) ? 2u : (b == 16) ? 3u : 0u; }

// Where the pad bytes behind the ten sections of a card start and how many there are (each fewer than 256).
// Built on the host and handed to the kernels, which only loop over it.
struct PadTable {
  uint64_t at[10];
  uint32_t len[10];
};

inline PadTable make_pad_table(const CardGeom& g) {
  PadTable t;
  const uint64_t T = g.tokens, P = g.planes, D = g.head_dim, M = (uint64_t)(g.head_dim / g.group_size) * 4;
  uint64_t start[10], used[10];
  start[0] = g.off_bits;  used[0] = T;
  start[1] = g.off_slot;  used[1] = 4ull * T;
  start[2] = g.off_order; used[2] = 4ull * T;
  for (int c = 0; c < 3; ++c) {
    start[3 + 2 * c] = g.off_codes[c]; used[3 + 2 * c] = P * g.n[c] * (D * width_of_class(c) / 8);
    start[4 + 2 * c] = g.off_meta[c];  used[4 + 2 * c] = P * g.n[c] * M;
  }
  start[9] = g.off_fp16; used[9] = P * g.n[3] * D * 2;
  for (int s = 0; s < 10; ++s) {
    t.at[s] = start[s] + used[s];
    t.len[s] = (uint32_t)(align256(used[s]) - used[s]);
  }
  return t;
}

// The 256 header bytes with `status` in place of the host's status word, and zeros in the pad
// bytes behind every section.  Call with tid = 0 .. 255 at least; every tid writes at most one
// header word and one byte per pad.
__device__ inline void write_header_and_pads(uint8_t* __restrict__ card, const qkv_card_header_t& header,
                                             const PadTable& pads, uint32_t status, uint32_t tid) {
  if (tid < 64) {
    const uint32_t* h = reinterpret_cast<const uint32_t*>(&header);
    uint32_t v = h[tid];
    if (tid == 48) v = status;                 // byte 192
    reinterpret_cast<uint32_t*>(card)[tid] = v;
  }
#pragma unroll
  for (int s = 0; s < 10; ++s)                  // unrolled: the table's loads are all in flight at once
    if (tid < pads.len[s]) card[pads.at[s] + tid] = 0;
}

}  // namespace qkv
